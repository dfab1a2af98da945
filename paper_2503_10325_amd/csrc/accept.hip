// Vocab-wide softmax statistics and the acceptance-rejection walk (Section 2.1 of the
// paper: accept x_i when q_i(x_i) <= o_i(x_i), else reject with probability
// 1 - o_i(x_i)/q_i(x_i); replacement from norm(max(0, o_i - q_i)); bonus token when
// nothing is rejected), extended to sibling drafts of a tree by recursive rejection.
//
// Kernels:
//   row_stats_kernel      one workgroup per (row, vocab segment): segment maximum and
//                         sum of 2^((l-m)c).  Pure streaming, HBM-bound.
//   accept_walk_kernel    one master workgroup per request: the sequential walk; every full
//                         pass over a row pair (residual mass, inverse-CDF search) is
//                         spread over the workgroup's 16 waves and, for large vocabularies,
//                         over the waves of up to three helper workgroups.
//   accept_linear_kernel  linear drafts: the scalar tests repeated in every workgroup, the one
//                         vocabulary-wide draw spread over several workgroups per request.
//   row_stats_prog_kernel large batches of linear drafts: the statistics pass in chain order, with
//                         the accept decisions taken on the way, so that rows behind a request's
//                         first rejection are not read.
// (accept_cluster.hip holds the tree kernel that reads only the rows a walk reaches.)
// Up to 128 draft nodes per request; the children of one node share one draft row, the one the
// first child names.
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

// (max, sum 2^((l - max) c)) of one 8192-logit segment of a row, by a workgroup of kStatThreads; the result is
// valid in thread 0, for which the function returns true.
template <bool VEC>
__device__ __forceinline__ bool segment_stats(const void* __restrict__ base, int dtype, int64_t row_off, int e_seg, int V,
                                              float c, float& M_out, double& Z_out) {
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
  double Z = 0.0;
#pragma unroll
  for (int w = 0; w < kStatThreads / kWave; ++w) Z += sh_z[w];
  M_out = M;
  Z_out = Z;
  return threadIdx.x == 0;
}

template <bool VEC>
__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(
    const void* __restrict__ t_base, int t_dtype, int n_t_rows,
    const void* __restrict__ q_base, int q_dtype, int n_q_rows,
    int V, float c, int nseg, SegStat* __restrict__ stats, unsigned* __restrict__ zero_words, int n_zero,
    const int32_t* __restrict__ q_row, int n_nodes) {
  const int seg = blockIdx.x;
  const int row = blockIdx.y;
  // side job of the first workgroup: clear the flags the walk kernel's workgroups exchange
  if (seg == 0 && row == 0)
    for (int i = threadIdx.x; i < n_zero; i += kStatThreads) zero_words[i] = 0u;
  const void* base = t_base;
  int dtype = t_dtype;
  int64_t r = row;
  if (row >= n_t_rows) {
    base = q_base; dtype = q_dtype; r = row - n_t_rows;
    // With more draft rows than draft nodes (several drafters per position) most rows are nobody's:
    // a row no node was drawn from (q_row, clamped as the walk clamps it) is not read at all.
    if (q_row) {
      int mine = 0;
      for (int i = threadIdx.x; i < n_nodes; i += kStatThreads)
        mine |= (min(max(q_row[i], 0), n_q_rows - 1) == static_cast<int>(r));
      if (!__syncthreads_or(mine)) return;
    }
  }
  const int64_t row_off = r * static_cast<int64_t>(V);
  float M;
  double Z;
  if (segment_stats<VEC>(base, dtype, row_off, seg * kStatSeg, V, c, M, Z)) {
    SegStat st;
    st.m = M; st.pad = 0.f; st.z = Z;
    stats[static_cast<int64_t>(row) * nseg + seg] = st;
  }
}

__global__ __launch_bounds__(kStatThreads) void zero_words_kernel(unsigned* __restrict__ words, int n) {
  for (int i = threadIdx.x; i < n; i += kStatThreads) words[i] = 0u;
}

void launch_row_stats(const void* t_base, int t_dtype, int n_t_rows, const void* q_base, int q_dtype,
                      int n_q_rows, int V, float c, SegStat* stats, hipStream_t stream, unsigned* zero_words,
                      int n_zero, const int32_t* q_row, int n_nodes) {
  const int rows = n_t_rows + n_q_rows;
  if (rows <= 0 || V <= 0) return;
  const int nseg = stats_segments(V);
  dim3 grid(nseg, rows);
  const bool vec = (V % 8 == 0) && aligned16(t_base) && aligned16(q_base);
  if (vec)
    hipLaunchKernelGGL(row_stats_kernel<true>, grid, dim3(kStatThreads), 0, stream, t_base, t_dtype,
                       n_t_rows, q_base, q_dtype, n_q_rows, V, c, nseg, stats, zero_words, n_zero, q_row, n_nodes);
  else
    hipLaunchKernelGGL(row_stats_kernel<false>, grid, dim3(kStatThreads), 0, stream, t_base, t_dtype,
                       n_t_rows, q_base, q_dtype, n_q_rows, V, c, nseg, stats, zero_words, n_zero, q_row, n_nodes);
}

// ----------------------------------------------------------------------------------
// walk
// ----------------------------------------------------------------------------------
constexpr int kWalkThreads = 1024;
constexpr int kWalkWaves = kWalkThreads / kWave;
constexpr int kMaxNodes = 128;
constexpr int kMaxBlocksPerSeg = 256;      // vocabularies up to 16 * 256 * 512 = 2M tokens

struct WalkRows {
  const void* t_base; int t_dtype; int64_t t_off; float t_m; double t_invz;   // target row
  const void* q_base; int q_dtype; int64_t q_off; float q_m; double q_invz;   // draft row
  int q_is_probs;
  int have_q;       // level 0 needs no draft row
};

// Weight of token class v at residual level L (L rejections so far at this node):
//   r_0 = p;  w_k = max(0, r_{k-1} - q);  r_k = w_k / R_k,  R_k = sum_v w_k(v).
// The weight of level L is w_L (unnormalised; p itself at level 0).  Per-class values are
// fp32 (their relative error, ~1e-7, is that of the hardware exp2 anyway); every sum over
// classes is carried in fp64.
// Weights of eight consecutive token classes from their logits (q: logits or probabilities).
// The level loop is outermost so that its (wave-uniform) trip count is tested once per eight classes;
// the last level stays unnormalised (scale 1, exact).
__device__ __forceinline__ void weights_from(const WalkRows& R, const float (&lp)[8], const float (&lq)[8],
                                             int n_valid, float c, int L, const float* __restrict__ inv_R,
                                             float (&w)[8]) {
  const float t_invz = static_cast<float>(R.t_invz), q_invz = static_cast<float>(R.q_invz);
  float q[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    w[j] = fast_exp2((lp[j] - R.t_m) * c) * t_invz;
    q[j] = 0.f;
    if (L > 0) q[j] = R.q_is_probs ? lq[j] : fast_exp2((lq[j] - R.q_m) * c) * q_invz;
  }
  for (int k = 0; k < L; ++k) {
    const float scale = (k + 1 < L) ? inv_R[k] : 1.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = fmaxf(w[j] - q[j], 0.f) * scale;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) w[j] = (j < n_valid) ? w[j] : 0.f;
}

template <bool VEC>
__device__ __forceinline__ void weights8(const WalkRows& R, int e0, int V, float c, int L,
                                         const float* __restrict__ inv_R, float (&w)[8]) {
  float lp[8], lq[8];
  load8<VEC>(R.t_base, R.t_dtype, R.t_off, e0, V, lp);
  if (L > 0) load8<VEC>(R.q_base, R.q_dtype, R.q_off, e0, V, lq);
  weights_from(R, lp, lq, min(8, V - e0), c, L, inv_R, w);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void unpack_bf16x8(u32x4 r, float (&x)[8]) {
  x[0] = bf16_lo(r[0]); x[1] = bf16_hi(r[0]); x[2] = bf16_lo(r[1]); x[3] = bf16_hi(r[1]);
  x[4] = bf16_lo(r[2]); x[5] = bf16_hi(r[2]); x[6] = bf16_lo(r[3]); x[7] = bf16_hi(r[3]);
}

// Sum of the level-L weights over [e_begin, e_end) (a multiple of 512 tokens wide, nit blocks) by one
// wave; the result is in every lane.  FAST: 16-byte aligned bf16 rows, four 512-token blocks in flight.
template <bool VEC, bool FAST>
__device__ __forceinline__ double wave_pass_sum(const WalkRows& R, int L, const float* __restrict__ inv_Rf,
                                                int e_begin, int e_end, int nit, int V, float c, int lane) {
  double acc = 0.0;
  if constexpr (FAST) {
    const uint16_t* tp = static_cast<const uint16_t*>(R.t_base) + R.t_off;
    const uint16_t* qp = static_cast<const uint16_t*>(R.q_base) + R.q_off;
    for (int it0 = 0; it0 < nit; it0 += 4) {
      u32x4 rp[4], rq[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e0 = min(e_begin + (it0 + u) * 512 + lane * 8, V - 8);     // clamped; masked below
        rp[u] = *reinterpret_cast<const u32x4*>(tp + e0);
        if (L > 0) rq[u] = *reinterpret_cast<const u32x4*>(qp + e0);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int it = it0 + u;
        if (it < nit) {
          const int e0 = e_begin + it * 512 + lane * 8;
          float lp[8], lq[8];
          unpack_bf16x8(rp[u], lp);
          if (L > 0) unpack_bf16x8(rq[u], lq);
          float w[8];
          weights_from(R, lp, lq, e0 < e_end ? 8 : 0, c, L, inv_Rf, w);
          float lsf = 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) lsf += w[j];
          acc += static_cast<double>(lsf);
        }
      }
    }
  } else {
    for (int it = 0; it < nit; ++it) {
      const int e0 = e_begin + it * 512 + lane * 8;
      float lsf = 0.f;
      if (e0 < e_end) {
        float w[8];
        weights8<VEC>(R, e0, V, c, L, inv_Rf, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) lsf += w[j];
      }
      acc += static_cast<double>(lsf);
    }
  }
  return wave_sum(acc);
}

// ---- helper workgroups -----------------------------------------------------------------------
// A full pass over a large vocabulary is bound by the vector ALU of the one compute unit that runs
// the request's walk (two exp2 per class).  For such vocabularies every request gets up to three
// helper workgroups on other compute units: the vocabulary is cut into 16 x (1 + helpers) contiguous
// wave segments, the master publishes what a pass needs, each helper sums its 16 segments and hands
// the sums back, and the master goes on as if it had 64 waves.  The partition is static and the
// grid (masters first, then helpers) is at most one workgroup per compute unit, so every workgroup
// becomes resident without waiting for another; helpers only ever wait for their master, the master
// only for its helpers, and every wait is bounded.
// Everything exchanged goes through relaxed device-scope atomic accesses (they bypass the
// non-coherent cache levels for exactly these words; acquire/release would write back and
// invalidate the whole L2 of the XCD on every poll and evict the logit rows the passes re-read).
// Order between a payload and its flag: the payload's stores have completed (vmcnt 0) before the
// flag is written.
template <typename T> __device__ __forceinline__ T ld_dev(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ void st_dev(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- pieces shared by the kernels that take the scalar accept decisions --------------------------------
// Merged (max, sum) of one logit row from its per-segment records, by a group of 16 lanes (lane sl of the
// group takes segments sl, sl + 16, ...); the result is in every lane of the group.  DEV: read the records
// with device-scope loads (they were written by other workgroups of the same kernel).  The arithmetic and
// its order are the same for every caller, so every caller gets the same bits.
template <bool DEV>
__device__ __forceinline__ void merged_row_stats(const SegStat* __restrict__ rec, int nseg, float c, int sl,
                                                 float& m_out, double& z_out) {
  auto load = [&](int sg) -> SegStat {
    if constexpr (DEV) {
      const unsigned long long* w = reinterpret_cast<const unsigned long long*>(rec + sg);
      const unsigned long long w0 = ld_dev(w), w1 = ld_dev(w + 1);
      SegStat st;
      st.m = __uint_as_float(static_cast<unsigned>(w0));
      st.pad = 0.f;
      st.z = __builtin_bit_cast(double, w1);
      return st;
    } else {
      return rec[sg];
    }
  };
  float m = -INFINITY;
  for (int sg = sl; sg < nseg; sg += 16) m = fmaxf(m, load(sg).m);
#pragma unroll
  for (int d = 8; d > 0; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 16));
  double z = 0.0;
  for (int sg = sl; sg < nseg; sg += 16) {
    const SegStat st = load(sg);
    if (st.m != -INFINITY) z += st.z * exp2(static_cast<double>(st.m - m) * static_cast<double>(c));
  }
#pragma unroll
  for (int d = 8; d > 0; d >>= 1) z += __shfl_xor(z, d, 16);
  m_out = m;
  z_out = z;
}

// r(x)/q(x) of a drafted token x at residual level 0 from its two logits and the merged row statistics
// (q: a logit, or the probability itself).  q(x) = 0 < p(x) accepts, q(x) = p(x) = 0 rejects.
__device__ __forceinline__ double accept_ratio(double lp, float t_m, double t_invz, double lq, float q_m, double q_invz,
                                               float c, bool q_is_probs) {
  const double px = exp2((lp - static_cast<double>(t_m)) * static_cast<double>(c)) * t_invz;
  const double qx = q_is_probs ? lq : exp2((lq - static_cast<double>(q_m)) * static_cast<double>(c)) * q_invz;
  if (qx > 0.0) return px / qx;
  return (px > 0.0) ? INFINITY : 0.0;
}

// ----------------------------------------------------------------------------------
// Statistics pass for large batches of linear drafts that stops reading a request's rows once its chain is known
// to have ended (Section 2.1: a rejection discards every later token).  Grid (segment, request, level), levels in
// the order the chain needs them: target row 0, then for node j = 0, 1, ... its draft row and target row j + 1.
// The 2 x nseg workgroups that produce the two rows of node j count their arrivals; the last one merges the two
// rows' statistics, gathers the node's two logits and takes the accept decision with the arithmetic the
// linear-draft kernel will use (same functions, same order: same bits); a rejection lowers stop[request] to j.
// A workgroup of a later level looks at stop[request] first and returns without reading when its row lies
// behind the stop.  Workgroups start roughly in grid order, so deep levels usually see the decisions of
// shallow ones; nothing depends on it - whatever was skipped lies behind the final stop, and the linear-draft
// kernel never uses a row behind its own first rejection, which is that same stop.
// ----------------------------------------------------------------------------------
constexpr int kProgMaxNodes = 64;
constexpr int kCntStride = 32;             // ints between two arrival counters: one 128-byte line each
constexpr int kProgStopStride = 32;        // ints between two requests' stop words: one 128-byte line each (every workgroup of a request reads its word)

__global__ __launch_bounds__(kStatThreads) void accept_prog_init_kernel(unsigned* __restrict__ node_cnt, int n_cnt,
                                                                       int* __restrict__ stop, unsigned* __restrict__ arrived, int B) {
  const int t = blockIdx.x * kStatThreads + threadIdx.x, nt = gridDim.x * kStatThreads;
  for (int i = t; i < n_cnt; i += nt) node_cnt[i * kCntStride] = 0u;
  for (int i = t; i < B; i += nt) { stop[i * kProgStopStride] = 0x7fffffff; arrived[i * kCntStride] = 0u; }
}

template <bool VEC>
__global__ __launch_bounds__(kStatThreads) void row_stats_prog_kernel(
    const void* __restrict__ t_base, int t_dtype, int n_t_rows, const void* __restrict__ q_base, int q_dtype, int n_q_rows,
    int V, float c, int nseg, SegStat* __restrict__ stats, const int32_t* __restrict__ node_offsets,
    const int32_t* __restrict__ q_row, const int32_t* __restrict__ draft_tokens, const float* __restrict__ u_accept,
    unsigned* __restrict__ node_cnt, int* __restrict__ stop, int max_nodes) {
  const int seg = blockIdx.x, b = blockIdx.y, k = blockIdx.z;
  const int tid = threadIdx.x;
  // (the three loads are independent: one round trip)
  const int st = ld_dev(stop + b * kProgStopStride);
  const int o = node_offsets[b];
  int n = node_offsets[b + 1] - o;
  n = n < 0 ? 0 : (n > max_nodes ? max_nodes : n);
  const bool is_q = (k & 1) != 0;
  const int j = is_q ? (k - 1) / 2 : k / 2 - 1;          // draft row of node j / target row j + 1 (k = 0: target row 0)
  if (k > 0 && j >= n) return;                           // the request has no such row
  if (k > 0 && (is_q ? st < j : st <= j)) return;        // the chain ended before this row is needed
  const int64_t trow0 = static_cast<int64_t>(o) + b;
  const void* base;
  int dtype;
  int64_t r, srow;
  if (is_q) {
    const int qr = min(max(q_row[o + j], 0), n_q_rows - 1);
    base = q_base; dtype = q_dtype; r = qr; srow = static_cast<int64_t>(n_t_rows) + qr;
  } else {
    base = t_base; dtype = t_dtype; r = trow0 + j + 1; srow = r;
  }
  float M;
  double Z;
  const bool writer = segment_stats<VEC>(base, dtype, r * static_cast<int64_t>(V), seg * kStatSeg, V, c, M, Z);
  // the node whose decision this row feeds: its own (draft row j) or the one tested against it (target row i: node i)
  const int node = is_q ? j : j + 1;
  if (tid >= kWave) return;           // what is left is one wave's work: the other waves free their slots now
  const int lane = tid;
  int last = 0;
  if (writer) {                       // lane 0
    unsigned long long* w = reinterpret_cast<unsigned long long*>(stats + srow * nseg + seg);
    st_dev(w, static_cast<unsigned long long>(__float_as_uint(M)));
    st_dev(w + 1, __builtin_bit_cast(unsigned long long, Z));
    if (node < n) {
      wait_stores();
      const unsigned old = __hip_atomic_fetch_add(&node_cnt[static_cast<int64_t>(o + node) * kCntStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      last = (old == static_cast<unsigned>(2 * nseg - 1));
    }
  }
  last = __shfl(last, 0, kWave);
  if (!last) return;
  // ---- both rows of `node` are complete: its accept decision, by this wave ----
  const int x = min(max(draft_tokens[o + node], 0), V - 1);
  const int qr = min(max(q_row[o + node], 0), n_q_rows - 1);
  float m = 0.f;
  double z = 1.0;
  {
    const int which = (lane >> 4) & 1, sl = lane & 15;   // lanes 0-15: the target row, 16-31: the draft row (32-63 repeat them)
    const int64_t sr = which ? static_cast<int64_t>(n_t_rows) + qr : trow0 + node;
    merged_row_stats<true>(stats + sr * nseg, nseg, c, sl, m, z);
  }
  const float m_t = __shfl(m, 0, kWave), m_q = __shfl(m, 16, kWave);
  const double z_t = __shfl(z, 0, kWave), z_q = __shfl(z, 16, kWave);
  if (lane == 0) {
    const double lp = static_cast<double>(load_logit(t_base, t_dtype, (trow0 + node) * static_cast<int64_t>(V) + x));
    const double lq = static_cast<double>(load_logit(q_base, q_dtype, static_cast<int64_t>(qr) * V + x));
    const double ratio = accept_ratio(lp, m_t, 1.0 / z_t, lq, m_q, 1.0 / z_q, c, false);
    if (!(static_cast<double>(u_accept[o + node]) < ratio))
      __hip_atomic_fetch_min(stop + b * kProgStopStride, node, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

constexpr int kMaxHelpers = 3;

// What a helper wave hands back: the sum of its segment and the pass it belongs to.  The wave
// writes the sum, waits for that store to complete, then writes the pass number; the master reads
// the 16 bytes with one load (one access to one cache line), so a matching pass number always comes
// with its sum and a hand-off costs a single trip.
struct __attribute__((aligned(16))) PartSlot {
  double sum;
  unsigned seq;
  unsigned pad;
};
__device__ __forceinline__ PartSlot ld_slot(const PartSlot* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  PartSlot r;
  r.sum = __builtin_bit_cast(double, (static_cast<unsigned long long>(v[1]) << 32) | v[0]);
  r.seq = v[2];
  r.pad = 0;
  return r;
}
constexpr unsigned kDone = 0xffffffffu;    // pass number that tells the helpers to leave
constexpr int kSpinLimit = 4000;           // a helper whose master never shows up leaves after this many polls (a few
                                           // milliseconds: ten times the master's own patience)

struct PassDesc {            // written by the master, published by `seq` (pass number, from 1)
  unsigned seq;
  int level;
  long long t_off, q_off;
  float t_m, q_m;
  double t_invz, q_invz;
  float inv_R[kMaxNodes];
};

struct AcceptParams {
  int B, V, n_t_rows, n_q_rows, nseg;
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
  int helpers;              // helper workgroups per request (0: the master works alone)
  int patience;             // polls a master spends on its helpers before it sums their segments itself
  PassDesc* desc;           // [B]
  PartSlot* part;           // [B][helpers][16] wave sums handed back by the helpers
};

// FAST: 16-byte aligned rows with both logit matrices in bf16 (the default layout): the full
// passes keep four 512-token blocks in flight per wave.
template <bool VEC, bool FAST>
__global__ __launch_bounds__(kWalkThreads) void accept_walk_kernel(AcceptParams P) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int S = P.helpers;
  const int vwaves = kWalkWaves * (1 + S);                 // wave segments the vocabulary is cut into
  __shared__ float sh_inv_Rf[kMaxNodes];     // 1 / R_k, fp32, for the per-class passes
  __shared__ unsigned sh_seq;
  __shared__ int sh_flag;

  // =============================== helper workgroup ===============================
  if (static_cast<int>(blockIdx.x) >= P.B) {
    const int idx = blockIdx.x - P.B;
    const int hb = idx % P.B, h = idx / P.B;               // request, helper number 0..S-1
    const int seg_w = (((P.V + vwaves - 1) / vwaves) + 511) / 512 * 512;
    const int e_begin = ((h + 1) * kWalkWaves + wave) * seg_w;
    const int e_end = min(P.V, e_begin + seg_w);
    const int nit = e_end > e_begin ? (e_end - e_begin + 511) / 512 : 0;
    PassDesc* desc = P.desc + hb;
    unsigned last_seq = 0;
    // Roles inside the loop are per wave, never per lane: with `if (tid == 0)` at the end of one
    // iteration and at the start of the next, the compiler routes the other lanes of wave 0 around
    // both, and they reach the workgroup barrier without lane 0 - a partial wave at s_barrier.
    // All 64 lanes of wave 0 poll (one coalesced load) and store the same words.
    for (;;) {
      if (wave == 0) {
        int spins = 0, fin = 0;
        unsigned seq = 0;
        for (;;) {
          seq = ld_dev(&desc->seq);                          // kDone once the master needs no more passes
          if (seq == kDone) { fin = 1; break; }
          if (seq > last_seq) break;
          __builtin_amdgcn_s_sleep(1);
          if (++spins > kSpinLimit) { fin = 1; break; }      // the master never came: leave
        }
        sh_seq = seq;
        sh_flag = fin;
      }
      __syncthreads();
      if (sh_flag) return;
      const unsigned seq = sh_seq;
      WalkRows R;
      R.t_base = P.target; R.t_dtype = P.t_dtype; R.q_base = P.draft_q; R.q_dtype = P.q_dtype;
      R.q_is_probs = (P.q_kind == 1); R.have_q = 1;
      const int level = ld_dev(&desc->level);
      R.t_off = ld_dev(&desc->t_off); R.q_off = ld_dev(&desc->q_off);
      R.t_m = ld_dev(&desc->t_m); R.q_m = ld_dev(&desc->q_m);
      R.t_invz = ld_dev(&desc->t_invz); R.q_invz = ld_dev(&desc->q_invz);
      sh_inv_Rf[tid & (kMaxNodes - 1)] = ld_dev(&desc->inv_R[tid & (kMaxNodes - 1)]);    // every thread, same values
      __syncthreads();
      // Normally the master rewrites the descriptor only after this helper has handed back the sums of
      // pass `seq`.  A master that ran out of patience may already be at a later pass: the copy above
      // can then mix two passes (every field is still a valid value of one of them, so all reads stay
      // in bounds) and the sum written below carries the old pass number, which the master ignores.
      const double acc = wave_pass_sum<VEC, FAST>(R, min(max(level, 0), kMaxNodes), sh_inv_Rf, e_begin, e_end, nit, P.V, P.c, lane);
      PartSlot* slot = P.part + (static_cast<int64_t>(hb) * S + h) * kWalkWaves + wave;
      st_dev(&slot->sum, acc);                   // all lanes of the wave store the same words
      wait_stores();
      st_dev(&slot->seq, seq);
      last_seq = seq;
      __syncthreads();                           // sh_inv_Rf and sh_seq are rewritten in the next round
    }
  }

  // =============================== master workgroup ===============================
  const int b = blockIdx.x;
  const int o = P.node_offsets[b];
  int n = P.node_offsets[b + 1] - o;
  n = n < 0 ? 0 : (n > kMaxNodes ? kMaxNodes : n);
  const int64_t trow0 = static_cast<int64_t>(o) + b;
  const int V = P.V;
  const float c = P.c;
  // contiguous vocab segment of each wave (the master's 16 and the helpers'), a multiple of 512 tokens
  const int seg_w = (((V + vwaves - 1) / vwaves) + 511) / 512 * 512;

  __shared__ double sh_wave_sum[kWalkWaves * (1 + kMaxHelpers)];
  __shared__ unsigned long long sh_missing;
  __shared__ double sh_blk[kMaxBlocksPerSeg];   // sums of the 512-token blocks of the segment the draw falls in
  __shared__ double sh_inv_R[kMaxNodes];     // 1 / R_k for the scalar accept tests
  __shared__ int sh_token;
  // per-request tables filled once, in parallel, so that the walk itself touches no global memory
  __shared__ float sh_tm[kMaxNodes + 1];       // target local row i: max logit
  __shared__ double sh_tinvz[kMaxNodes + 1];   //                     1 / sum 2^((l-m)c)
  __shared__ float sh_qm[kMaxNodes];           // draft row of node j
  __shared__ double sh_qinvz[kMaxNodes];
  __shared__ int sh_par[kMaxNodes], sh_tok[kMaxNodes], sh_qrow[kMaxNodes];
  __shared__ double sh_px[kMaxNodes], sh_qx[kMaxNodes];   // p_parent(x_j), q(x_j)
  __shared__ float sh_u[kMaxNodes];
  __shared__ int sh_fc[kMaxNodes + 1];         // first child (lowest index) of node i at [i + 1]

  const bool q_is_probs = (P.q_kind == 1);
  const double u_res = static_cast<double>(P.u_resample[b]);      // needed last; fetched first
  // (1) node arrays
  if (tid <= kMaxNodes) sh_fc[tid] = kMaxNodes;
  if (tid < n) {
    int par = P.parent ? P.parent[o + tid] : tid - 1;
    if (par < -1 || par >= tid) par = -1;
    sh_par[tid] = par;
    // indices come from device memory the host cannot check: clamp them so that a bad entry
    // gives a wrong answer for that request instead of an out-of-bounds read
    sh_tok[tid] = min(max(P.draft_tokens[o + tid], 0), V - 1);
    sh_qrow[tid] = min(max(P.q_row[o + tid], 0), P.n_q_rows - 1);
    sh_u[tid] = P.u_accept[o + tid];
    if (P.dbg_ratio) P.dbg_ratio[o + tid] = __builtin_nanf("");
  }
  if (tid < kMaxNodes) sh_inv_Rf[tid] = 0.f;
  __syncthreads();
  if (P.parent) {
    // The children of one node were drawn from one draft distribution: the row its first child names.  Every
    // sibling uses that row (for q(x) and for the residual), whatever its own q_row entry says.
    if (tid < n) atomicMin(&sh_fc[sh_par[tid] + 1], tid);
    __syncthreads();
    int group_row = 0;
    if (tid < n) group_row = sh_qrow[min(sh_fc[sh_par[tid] + 1], kMaxNodes - 1)];
    __syncthreads();
    if (tid < n) sh_qrow[tid] = group_row;
    __syncthreads();
  }
  // (2) in one round trip: the two logits of every drafted token (last wave) and the merged
  // statistics of the n+1 target rows and n draft rows (groups of 16 lanes, one segment each)
  if (wave == kWalkWaves - 1) {
    for (int j = lane; j < n; j += kWave) {
      const int x = sh_tok[j];
      sh_px[j] = static_cast<double>(load_logit(P.target, P.t_dtype, (trow0 + 1 + sh_par[j]) * static_cast<int64_t>(V) + x));
      sh_qx[j] = static_cast<double>(load_logit(P.draft_q, P.q_dtype, static_cast<int64_t>(sh_qrow[j]) * V + x));
    }
  } else {
    const int n_rows = (n + 1) + (q_is_probs ? 0 : n);
    const int sl = tid & 15;
    for (int ri = tid >> 4; ri < n_rows; ri += (kWalkThreads - kWave) / 16) {
      const int64_t srow = (ri <= n) ? trow0 + ri : static_cast<int64_t>(P.n_t_rows) + sh_qrow[ri - n - 1];
      float m = -INFINITY;
      for (int sg = sl; sg < P.nseg; sg += 16) m = fmaxf(m, P.stats[srow * P.nseg + sg].m);
#pragma unroll
      for (int d = 8; d > 0; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 16));
      double z = 0.0;
      for (int sg = sl; sg < P.nseg; sg += 16) {
        const SegStat st = P.stats[srow * P.nseg + sg];
        if (st.m != -INFINITY) z += st.z * exp2(static_cast<double>(st.m - m) * static_cast<double>(c));
      }
#pragma unroll
      for (int d = 8; d > 0; d >>= 1) z += __shfl_xor(z, d, 16);
      if (sl == 0) {
        if (ri <= n) { sh_tm[ri] = m; sh_tinvz[ri] = 1.0 / z; }
        else { sh_qm[ri - n - 1] = m; sh_qinvz[ri - n - 1] = 1.0 / z; }
      }
    }
  }
  __syncthreads();
  // (3) p(x), q(x) of every node
  if (tid < n) {
    const int par = sh_par[tid];
    sh_px[tid] = exp2((sh_px[tid] - static_cast<double>(sh_tm[par + 1])) * static_cast<double>(c)) * sh_tinvz[par + 1];
    if (!q_is_probs)
      sh_qx[tid] = exp2((sh_qx[tid] - static_cast<double>(sh_qm[tid])) * static_cast<double>(c)) * sh_qinvz[tid];
  }
  __syncthreads();

  // lane l looks after nodes l and l + 64; nodes that do not exist hold an impossible parent
  const int my_parent = (lane < n) ? sh_par[lane] : -2;
  const int my_parent_hi = (lane + kWave < n) ? sh_par[lane + kWave] : -2;

  int cur = -1, depth = 0;
  WalkRows R;
  R.t_base = P.target; R.t_dtype = P.t_dtype;
  R.q_base = P.draft_q; R.q_dtype = P.q_dtype; R.q_is_probs = q_is_probs;
  R.t_off = 0; R.t_m = 0.f; R.t_invz = 0.0;
  R.q_off = 0; R.q_m = 0.f; R.q_invz = 0.0; R.have_q = 0;

  const int e_begin = wave * seg_w;
  const int e_end = min(V, e_begin + seg_w);
  const int nit = e_end > e_begin ? (e_end - e_begin + 511) / 512 : 0;

  // One full pass at residual level L: per-wave sums (the master's and the helpers') to LDS, returns
  // the total.
  unsigned pass_no = 0;
  auto full_pass = [&](int L) -> double {
    __syncthreads();                 // previous readers of the sums are done
    ++pass_no;
    if (S > 0 && wave == 0) {          // all lanes of wave 0 store the same words (no per-lane role, see the helper loop)
      PassDesc* desc = P.desc + b;
      st_dev(&desc->level, L);
      st_dev(&desc->t_off, static_cast<long long>(R.t_off)); st_dev(&desc->q_off, static_cast<long long>(R.q_off));
      st_dev(&desc->t_m, R.t_m); st_dev(&desc->q_m, R.q_m);
      st_dev(&desc->t_invz, R.t_invz); st_dev(&desc->q_invz, R.q_invz);
      for (int k = 0; k < L && k < kMaxNodes; ++k) st_dev(&desc->inv_R[k], sh_inv_Rf[k]);
      wait_stores();
      st_dev(&desc->seq, pass_no);
    }
    const double acc = wave_pass_sum<VEC, FAST>(R, L, sh_inv_Rf, e_begin, e_end, nit, V, c, lane);
    if (lane == 0) sh_wave_sum[wave] = acc;
    if (S > 0) {
      if (wave == 0) {               // lane l watches helper wave l (the last one again for lanes beyond)
        const int n_slots = S * kWalkWaves;                     // <= 48
        const int my = min(lane, n_slots - 1);
        const PartSlot* slot = P.part + static_cast<int64_t>(b) * n_slots + my;
        int spins = 0;
        PartSlot got;
        bool up;
        for (;;) {
          got = ld_slot(slot);
          up = got.seq == pass_no;
          if (__all(up)) break;
          if (++spins > P.patience) break;                      // helpers not there (yet): see below
          __builtin_amdgcn_s_sleep(1);
        }
        if (up) sh_wave_sum[kWalkWaves + my] = got.sum;         // lanes beyond n_slots repeat the last slot
        const unsigned long long missing = __ballot(!up) & ((1ull << n_slots) - 1ull);
        if (lane == 0) sh_missing = missing;
      }
      __syncthreads();
      // Segments whose helper wave has not answered within the patience (its workgroup may not be
      // resident yet when other kernels fill the GPU) are summed here instead: the walk never
      // depends on a helper making progress.  A late answer is ignored (its pass number is old).
      unsigned long long miss = sh_missing;
      for (int k = 0; miss; ++k) {
        const int j = __ffsll(static_cast<long long>(miss)) - 1;
        miss &= miss - 1;
        if ((k & (kWalkWaves - 1)) != wave) continue;
        const int hb_begin = (kWalkWaves + j) * seg_w;
        const int hb_end = min(V, hb_begin + seg_w);
        const int hb_nit = hb_end > hb_begin ? (hb_end - hb_begin + 511) / 512 : 0;
        const double a2 = wave_pass_sum<VEC, FAST>(R, L, sh_inv_Rf, hb_begin, hb_end, hb_nit, V, c, lane);
        if (lane == 0) sh_wave_sum[kWalkWaves + j] = a2;
      }
    }
    __syncthreads();
    double tot = 0.0;
    for (int w = 0; w < vwaves; ++w) tot += sh_wave_sum[w];
    return tot;
  };

  int level = 0;          // rejections so far at the current node
  int sums_level = -1;    // level whose sums sit in LDS (-1: none)
  double total = 0.0;     // total of those sums

  for (int guard = 0; guard <= kMaxNodes; ++guard) {
    // target row of the current node
    R.t_off = (trow0 + 1 + cur) * static_cast<int64_t>(V);
    R.t_m = sh_tm[cur + 1];
    R.t_invz = sh_tinvz[cur + 1];
    level = 0;
    sums_level = -1;
    R.have_q = 0;

    // children of the current node in index order: two ballot words
    unsigned long long kids = __ballot(my_parent == cur && lane > cur);
    unsigned long long kids_hi = __ballot(my_parent_hi == cur && lane + kWave > cur);
    int accepted = -1;
    while (kids | kids_hi) {
      int ch;
      if (kids) { ch = __ffsll(static_cast<long long>(kids)) - 1; kids &= kids - 1; }
      else { ch = kWave + __ffsll(static_cast<long long>(kids_hi)) - 1; kids_hi &= kids_hi - 1; }
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
        if (tid == 0) { sh_inv_R[level] = 1.0 / mass; sh_inv_Rf[level] = static_cast<float>(1.0 / mass); }
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
    if (S > 0 && wave == 0) st_dev(&P.desc[b].seq, kDone);  // no more passes: the helpers may leave
    const double target = u_res * total;
    int ws = -1;
    double before = 0.0;
    for (int w = 0; w < vwaves; ++w) {
      const double sw = sh_wave_sum[w];
      if (before + sw > target) { ws = w; break; }
      before += sw;
    }
    if (ws < 0) {                    // rounding left no crossing: last wave segment with positive mass
      for (int w = vwaves - 1; w >= 0; --w) if (sh_wave_sum[w] > 0.0) { ws = w; break; }
      if (ws < 0) ws = 0;
      before = 0.0;
      for (int w = 0; w < ws; ++w) before += sh_wave_sum[w];
    }
    // block of 512 tokens inside segment ws: the 16 waves sum its blocks in parallel
    const int ws_begin = ws * seg_w;
    const int ws_end = min(V, ws_begin + seg_w);
    const int ws_nit = ws_end > ws_begin ? (ws_end - ws_begin + 511) / 512 : 0;
    __syncthreads();
    for (int it = wave; it < ws_nit; it += kWalkWaves) {
      const int e0 = ws_begin + it * 512 + lane * 8;
      float lsf = 0.f;
      if (e0 < ws_end) {
        float w[8];
        weights8<VEC>(R, e0, V, c, level, sh_inv_Rf, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) lsf += w[j];
      }
      const double ls = wave_sum(static_cast<double>(lsf));
      if (lane == 0) sh_blk[it] = ls;
    }
    __syncthreads();
    const double* blk = sh_blk;
    int it_hit = -1;
    double run = before;
    for (int it = 0; it < ws_nit; ++it) {
      const double sblk = blk[it];
      if (run + sblk > target) { it_hit = it; break; }
      run += sblk;
    }
    if (it_hit < 0) {                // rounding: last block of the segment with positive mass
      for (int it = ws_nit - 1; it >= 0; --it) if (blk[it] > 0.0) { it_hit = it; break; }
      if (it_hit < 0) it_hit = 0;
      run = before;
      for (int it = 0; it < it_hit; ++it) run += blk[it];
    }
    if (wave == 0) {
      const int e0 = ws_begin + it_hit * 512 + lane * 8;
      float w[8];
      if (e0 < ws_end) weights8<VEC>(R, e0, V, c, level, sh_inv_Rf, w);
      else {
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = 0.f;
      }
      float lsf = 0.f;                 // summed exactly as the pass did, so the block sums agree
      int my_last = -1;
#pragma unroll
      for (int j = 0; j < 8; ++j) { lsf += w[j]; if (w[j] > 0.f) my_last = e0 + j; }
      const double ls = static_cast<double>(lsf);
      double inc = ls;                 // inclusive scan of the lane sums
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const double tq = __shfl_up(inc, d, kWave);
        if (lane >= d) inc += tq;
      }
      const unsigned long long cross = __ballot(run + inc > target);
      int found = -1;
      if (cross) {
        const int fl = __ffsll(static_cast<long long>(cross)) - 1;
        // every lane works out its own candidate: no lane-dependent branch ahead of the broadcast
        // (with one, the compiler may let lanes reach the broadcast without the lane they read from)
        int tok = -1;
        double acc = run + inc - ls;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          acc += static_cast<double>(w[j]);
          if (tok < 0 && acc > target && w[j] > 0.f) tok = e0 + j;
        }
        if (tok < 0) tok = my_last;        // rounding inside the lane: its last positive class
        found = __shfl(tok, fl, kWave);
      }
      if (found < 0) {                     // rounding across lanes: last positive class of the block
        int ml = my_last;
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) ml = max(ml, __shfl_xor(ml, d, kWave));
        found = ml >= 0 ? ml : min(V - 1, ws_begin + it_hit * 512);
      }
      if (lane == 0 && depth < P.out_stride) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + depth] = found;
    }
    break;
  }
  if (tid == 0) {
    if (S > 0) st_dev(&P.desc[b].seq, kDone);
    P.accept_len[b] = depth;
    if (P.stop_node) P.stop_node[b] = cur;
  }
  for (int i = depth + 1 + tid; i < P.out_stride; i += kWalkThreads) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + i] = -1;
}

// ----------------------------------------------------------------------------------
// Linear drafts (no parent array): a chain is rejected at most once, so after the scalar accept tests exactly one
// vocabulary-wide distribution is left to draw from - max(0, p - q) of the rejected position, or p after the
// last draft when nothing was rejected (Section 2.1).  accept_linear_kernel spreads that one pass over the chip:
// a unit of one to four 4096-class blocks per workgroup, U workgroups per request.  Every workgroup repeats the
// request's scalar tests (a few dozen values from the row statistics), sums the weights of its blocks and hands
// the block sums over; the workgroup that arrives last adds them, finds the block of the draw and re-reads that
// block alone for the class.  Nobody waits for anybody.
// ----------------------------------------------------------------------------------
constexpr int kLinThreads = 512;
constexpr int kLinWaves = kLinThreads / kWave;
constexpr int kLinBlock = kLinThreads * 8;         // classes one sweep of a workgroup covers
constexpr int kLinMaxBlocks = 4;                   // blocks per unit at most (their loads are issued together)
constexpr int kLinMaxUnits = 512;                  // vocabularies up to 2M classes

// most units a vocabulary can be cut into (one block each): sizes the workspace
int linear_units(int V) { return (V + kLinBlock - 1) / kLinBlock; }

// Classes per workgroup (whole blocks): about two workgroups per compute unit for the whole batch.
static int linear_unit_classes(int B, int V, int n_cu) {
  const int max_units = linear_units(V);
  int U = (2 * n_cu + B - 1) / (B > 0 ? B : 1);
  const int min_units = (max_units + kLinMaxBlocks - 1) / kLinMaxBlocks;
  U = U < min_units ? min_units : (U > max_units ? max_units : U);
  const int per = (V + U - 1) / U;
  return (per + kLinBlock - 1) / kLinBlock * kLinBlock;
}

template <bool VEC>
__global__ __launch_bounds__(kLinThreads, 2) void accept_linear_kernel(AcceptParams P, double* __restrict__ partial,
                                                                    unsigned* __restrict__ arrived, int U, int unit_classes) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x / U, unit = blockIdx.x % U;
  const int o = P.node_offsets[b];
  int n = P.node_offsets[b + 1] - o;
  n = n < 0 ? 0 : (n > kMaxNodes ? kMaxNodes : n);
  const int64_t trow0 = static_cast<int64_t>(o) + b;
  const int V = P.V;
  const float c = P.c;
  const bool q_is_probs = (P.q_kind == 1);

  __shared__ float sh_tm[kMaxNodes + 1];
  __shared__ double sh_tinvz[kMaxNodes + 1];
  __shared__ float sh_qm[kMaxNodes];
  __shared__ double sh_qinvz[kMaxNodes];
  __shared__ int sh_tok[kMaxNodes], sh_qrow[kMaxNodes];
  __shared__ double sh_px[kMaxNodes], sh_qx[kMaxNodes];
  __shared__ float sh_u[kMaxNodes];
  __shared__ float sh_zero[kMaxNodes];           // 1/R_k of lower levels: none exist at levels 0 and 1
  __shared__ double sh_wsum[kLinWaves];
  __shared__ double sh_part[kLinMaxUnits];
  __shared__ int sh_last;
  __shared__ int sh_cross[kLinWaves], sh_lastpos[kLinWaves];
  __shared__ double sh_bw[kLinMaxBlocks][kLinWaves];

  const double u_res = static_cast<double>(P.u_resample[b]);
  // (1) node arrays (indices clamped: a bad entry gives a wrong answer for that request, never a wild read)
  if (tid < n) {
    sh_tok[tid] = min(max(P.draft_tokens[o + tid], 0), V - 1);
    sh_qrow[tid] = min(max(P.q_row[o + tid], 0), P.n_q_rows - 1);
    sh_u[tid] = P.u_accept[o + tid];
  }
  if (tid < kMaxNodes) sh_zero[tid] = 0.f;
  __syncthreads();
  // (2) the two logits of every drafted token (last wave) and the merged statistics of the n+1 target rows and
  // the n draft rows (groups of 16 lanes, one segment each)
  if (wave == kLinWaves - 1) {
    for (int j = lane; j < n; j += kWave) {
      const int x = sh_tok[j];
      sh_px[j] = static_cast<double>(load_logit(P.target, P.t_dtype, (trow0 + j) * static_cast<int64_t>(V) + x));
      sh_qx[j] = static_cast<double>(load_logit(P.draft_q, P.q_dtype, static_cast<int64_t>(sh_qrow[j]) * V + x));
    }
  } else {
    const int n_rows = (n + 1) + (q_is_probs ? 0 : n);
    const int sl = tid & 15;
    for (int ri = tid >> 4; ri < n_rows; ri += (kLinThreads - kWave) / 16) {
      const int64_t srow = (ri <= n) ? trow0 + ri : static_cast<int64_t>(P.n_t_rows) + sh_qrow[ri - n - 1];
      float m;
      double z;
      merged_row_stats<false>(P.stats + srow * P.nseg, P.nseg, c, sl, m, z);
      if (sl == 0) {
        if (ri <= n) { sh_tm[ri] = m; sh_tinvz[ri] = 1.0 / z; }
        else { sh_qm[ri - n - 1] = m; sh_qinvz[ri - n - 1] = 1.0 / z; }
      }
    }
  }
  __syncthreads();
  // (3) p(x_j), q(x_j) of every node in parallel (node j is tested against target row j, the distribution
  // after nodes 0..j-1), then the chain itself on LDS data
  __shared__ double sh_ratio[kMaxNodes];
  if (tid < n)
    sh_ratio[tid] = accept_ratio(sh_px[tid], sh_tm[tid], sh_tinvz[tid], sh_qx[tid], q_is_probs ? 0.f : sh_qm[tid],
                                 q_is_probs ? 0.0 : sh_qinvz[tid], c, q_is_probs);
  __syncthreads();
  int depth = 0, rejected = -1;
  for (int j = 0; j < n; ++j) {
    if (static_cast<double>(sh_u[j]) < sh_ratio[j]) { ++depth; continue; }
    rejected = j;
    break;
  }
  if (unit == 0 && P.dbg_ratio)
    for (int j = tid; j < n; j += kLinThreads)
      P.dbg_ratio[o + j] = (rejected < 0 || j <= rejected) ? static_cast<float>(sh_ratio[j]) : __builtin_nanf("");
  if (unit == 0) {          // everything but the drawn token is known here
    for (int i = tid; i < P.out_stride; i += kLinThreads)
      if (i != depth) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + i] = (i < depth) ? sh_tok[i] : -1;
    if (tid == 0) {
      P.accept_len[b] = depth;
      if (P.stop_node) P.stop_node[b] = depth - 1;
    }
  }
  WalkRows R;
  R.t_base = P.target; R.t_dtype = P.t_dtype;
  R.q_base = P.draft_q; R.q_dtype = P.q_dtype; R.q_is_probs = q_is_probs;
  R.t_off = (trow0 + depth) * static_cast<int64_t>(V);
  R.t_m = sh_tm[depth]; R.t_invz = sh_tinvz[depth];
  R.have_q = rejected >= 0;
  R.q_off = 0; R.q_m = 0.f; R.q_invz = 0.0;
  int level = 0;
  if (rejected >= 0) {
    R.q_off = static_cast<int64_t>(sh_qrow[rejected]) * V;
    if (!q_is_probs) { R.q_m = sh_qm[rejected]; R.q_invz = sh_qinvz[rejected]; }
    level = 1;
  }

  // Weights of this thread's eight classes in each block of unit k (at most kLinMaxBlocks blocks, their loads
  // issued together) and the per-block fp32 sums.  Identical arithmetic wherever it is called.
  const int bpu = unit_classes / kLinBlock;         // blocks per unit, <= kLinMaxBlocks
  const int nblocks = (V + kLinBlock - 1) / kLinBlock;
  auto unit_weights = [&](int k, int L, float (&w)[kLinMaxBlocks][8], float (&lsf)[kLinMaxBlocks]) {
    float lp[kLinMaxBlocks][8], lq[kLinMaxBlocks][8];
#pragma unroll
    for (int i = 0; i < kLinMaxBlocks; ++i) {
      const int e0 = (k * bpu + i) * kLinBlock + tid * 8;
      if (i < bpu && e0 < V) {
        load8<VEC>(R.t_base, R.t_dtype, R.t_off, e0, V, lp[i]);
        if (L > 0) load8<VEC>(R.q_base, R.q_dtype, R.q_off, e0, V, lq[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < kLinMaxBlocks; ++i) {
      const int e0 = (k * bpu + i) * kLinBlock + tid * 8;
      lsf[i] = 0.f;
      if (i < bpu && e0 < V) {
        weights_from(R, lp[i], lq[i], min(8, V - e0), c, L, sh_zero, w[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) lsf[i] += w[i][j];
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) w[i][j] = 0.f;
      }
    }
  };
  // per-block totals from the per-thread sums: fp64 across lanes and waves in a fixed order; in every thread
  auto block_totals = [&](const float (&lsf)[kLinMaxBlocks], double (&tot)[kLinMaxBlocks]) {
    __syncthreads();                  // earlier readers of sh_bw are done
#pragma unroll
    for (int i = 0; i < kLinMaxBlocks; ++i) {
      const double ws = wave_sum(static_cast<double>(lsf[i]));
      if (lane == 0) sh_bw[i][wave] = ws;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kLinMaxBlocks; ++i) {
      tot[i] = 0.0;
#pragma unroll
      for (int v = 0; v < kLinWaves; ++v) tot[i] += sh_bw[i][v];
    }
  };

  float w[kLinMaxBlocks][8], lsf[kLinMaxBlocks];
  double tot[kLinMaxBlocks];
  unit_weights(unit, level, w, lsf);
  block_totals(lsf, tot);
  if (wave == 0) {                    // all lanes of wave 0 store the same words (no per-lane role around barriers)
#pragma unroll
    for (int i = 0; i < kLinMaxBlocks; ++i)
      if (i < bpu && unit * bpu + i < nblocks) st_dev(&partial[static_cast<int64_t>(b) * nblocks + unit * bpu + i], tot[i]);
    wait_stores();
    unsigned old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(&arrived[b * kCntStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    sh_last = (old == static_cast<unsigned>(U - 1));
  }
  __syncthreads();
  if (!sh_last) return;

  // ---- the last workgroup of the request: total, block of the draw, class ----
  for (int k = tid; k < nblocks; k += kLinThreads) sh_part[k] = ld_dev(&partial[static_cast<int64_t>(b) * nblocks + k]);
  __syncthreads();
  double total = 0.0;
  for (int k = 0; k < nblocks; ++k) total += sh_part[k];
  if (level == 1 && !(total > 0.0)) {
    // a residual without mass leaves the distribution as it was: draw from p (sums redone here; rare)
    level = 0;
    R.have_q = 0;
    for (int k = 0; k < U; ++k) {
      unit_weights(k, 0, w, lsf);
      block_totals(lsf, tot);
      __syncthreads();
      if (tid == 0) {
#pragma unroll
        for (int i = 0; i < kLinMaxBlocks; ++i)
          if (i < bpu && k * bpu + i < nblocks) sh_part[k * bpu + i] = tot[i];
      }
    }
    __syncthreads();
    total = 0.0;
    for (int k = 0; k < nblocks; ++k) total += sh_part[k];
  }
  const double target = u_res * total;
  int kb_hit = -1;
  double before = 0.0;
  for (int k = 0; k < nblocks; ++k) {
    const double sk = sh_part[k];
    if (before + sk > target) { kb_hit = k; break; }
    before += sk;
  }
  if (kb_hit < 0) {                   // rounding left no crossing: last block with positive mass
    for (int k = nblocks - 1; k >= 0; --k) if (sh_part[k] > 0.0) { kb_hit = k; break; }
    if (kb_hit < 0) kb_hit = 0;
    before = 0.0;
    for (int k = 0; k < kb_hit; ++k) before += sh_part[k];
  }
  // that block alone: this thread's eight weights, the wave sums in LDS
  float wh[8];
  float lsh = 0.f;
  {
    const int eb = kb_hit * kLinBlock + tid * 8;
    if (eb < V) {
      weights8<VEC>(R, eb, V, c, level, sh_zero, wh);
#pragma unroll
      for (int j = 0; j < 8; ++j) lsh += wh[j];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) wh[j] = 0.f;
    }
    const double ws = wave_sum(static_cast<double>(lsh));
    __syncthreads();                  // earlier readers of sh_bw are done
    if (lane == 0) sh_bw[0][wave] = ws;
    __syncthreads();
  }
  const int e0 = kb_hit * kLinBlock + tid * 8;
  int my_last = -1;
#pragma unroll
  for (int j = 0; j < 8; ++j) if (wh[j] > 0.f) my_last = e0 + j;
  const double ls = static_cast<double>(lsh);
  double inc = ls;                    // inclusive scan of the lane sums inside the wave
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const double tq = __shfl_up(inc, d, kWave);
    if (lane >= d) inc += tq;
  }
  double run = before;                // mass ahead of this wave
  for (int v = 0; v < wave; ++v) run += sh_bw[0][v];
  const unsigned long long cross = __ballot(run + inc > target);
  int tok = -1;
  {
    double acc = run + inc - ls;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      acc += static_cast<double>(wh[j]);
      if (tok < 0 && acc > target && wh[j] > 0.f) tok = e0 + j;
    }
    if (tok < 0) tok = my_last;       // rounding inside the lane: its last positive class
  }
  const int fl = cross ? __ffsll(static_cast<long long>(cross)) - 1 : 0;
  const int cand = __shfl(tok, fl, kWave);
  int ml = my_last;
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) ml = max(ml, __shfl_xor(ml, d, kWave));
  if (lane == 0) { sh_cross[wave] = cross ? cand : -2; sh_lastpos[wave] = ml; }
  __syncthreads();
  if (tid == 0) {
    int found = -1;
    for (int v = 0; v < kLinWaves && found < 0; ++v)
      if (sh_cross[v] != -2) found = sh_cross[v];          // first wave with a crossing (-1: its lane had no positive class)
    if (found < 0) {                  // rounding across the block: its last positive class
      for (int v = kLinWaves - 1; v >= 0 && found < 0; --v) if (sh_lastpos[v] >= 0) found = sh_lastpos[v];
      if (found < 0) found = min(V - 1, kb_hit * kLinBlock);
    }
    if (depth < P.out_stride) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + depth] = found;
  }
}

// Workspace: [row statistics][helper protocol: pass descriptors, hand-back slots (zeroed by the
// statistics kernel)]
struct AcceptLayout {
  size_t words_off, n_zero_words, desc_off, part_off, arrived_off, msg_off, lin_off, prog_cnt_off, prog_stop_off, total;
};

static AcceptLayout accept_layout(int B, int total_nodes, int n_q_rows, int V) {
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  AcceptLayout l;
  const size_t rows = static_cast<size_t>(total_nodes) + B + n_q_rows;
  l.words_off = up(rows * stats_segments(V) * sizeof(SegStat));
  l.desc_off = l.words_off;
  l.part_off = l.desc_off + up(static_cast<size_t>(B) * sizeof(PassDesc));
  l.arrived_off = l.part_off + up(static_cast<size_t>(B) * kMaxHelpers * kWalkWaves * sizeof(PartSlot));
  l.msg_off = l.arrived_off + up(static_cast<size_t>(B) * kCntStride * sizeof(unsigned));   // arrival counters of the linear-draft kernel
  l.n_zero_words = (l.msg_off - l.words_off) / sizeof(unsigned);         // flags, descriptors, hand-back slots, counters
  l.lin_off = l.msg_off + up(cluster_msg_bytes(B));                      // messages of the cluster path
  l.prog_cnt_off = l.lin_off + up(static_cast<size_t>(B) * linear_units(V) * sizeof(double));   // block sums of the linear-draft kernel
  l.prog_stop_off = l.prog_cnt_off + up(static_cast<size_t>(total_nodes) * kCntStride * sizeof(unsigned));   // arrivals per node
  l.total = l.prog_stop_off + up(static_cast<size_t>(B) * kProgStopStride * sizeof(int)) + 256;      // first rejection per request
  return l;
}

size_t accept_workspace_bytes(int B, int total_nodes, int n_q_rows, int V) {
  return accept_layout(B, total_nodes, n_q_rows, V).total;
}

// Where the cluster path wins (measured): every 8192-logit unit of a row gets a compute unit of its own and
// the rows are long.  Short rows and batches with few compute units per request are faster through the
// statistics pass over all rows, whose arithmetic spreads over the whole chip.
static bool cluster_pays(int B, int V, int n_cu) {
  const int units = (V + 8191) / 8192;
  return units >= 8 && units <= 32 && static_cast<int64_t>(B) * units <= n_cu;
}

// Linear drafts take the statistics pass and accept_linear_kernel unless the caller asks for another path.
static bool linear_path(const AcceptArgs& a) {
  return a.parent == nullptr && (a.path == 0 || a.path == 3 || a.path == 4) && linear_units(a.V) <= kLinMaxUnits;
}

// The statistics pass that stops at each request's first rejection pays when the launch is several times what
// the chip holds at once (about 2048 workgroups): later levels then start after the decisions of earlier ones.
// It needs draft logits (their statistics are part of the decision) and computes the target rows itself.
static bool progressive_stats(const AcceptArgs& a) {
  if (!linear_path(a) || a.q_kind != 0 || a.target_stats_ready || a.total_nodes <= 0) return false;
  if (a.max_nodes > kProgMaxNodes || a.B > 65535) return false;
  const int64_t wgs = (static_cast<int64_t>(a.total_nodes) * 2 + a.B) * stats_segments(a.V);
  return a.path == 4 || (a.path == 0 && wgs >= 6144);
}

const char* accept_plan_name(const AcceptArgs& a, int n_cu) {
  const bool vec = (a.V % 8 == 0) && aligned16(a.target) && aligned16(a.draft_q);
  const bool cluster_ok = vec && a.V >= 8 && a.V <= kClusterMaxV && a.t_dtype == kBF16 && a.q_dtype == kBF16 &&
                          a.q_kind == 0;
  const bool cluster = cluster_ok && (a.path == 2 || (a.path == 0 && a.parent != nullptr && cluster_pays(a.B, a.V, n_cu)));
  if (!cluster && progressive_stats(a)) return "row_stats_prog_kernel (rows up to each request's first rejection) + accept_linear_kernel (linear drafts: one vocabulary unit per workgroup, the last to arrive draws)";
  if (!cluster && linear_path(a)) return "row_stats_kernel (all rows) + accept_linear_kernel (linear drafts: one vocabulary unit per workgroup, the last to arrive draws)";
  if (!cluster) return "row_stats_kernel (all rows) + accept_walk_kernel (one workgroup per request, helper workgroups)";
  const ClusterPlan p = make_cluster_plan(a.B, a.V, a.max_nodes, a.parent != nullptr, n_cu, a.levels, a.slices);
  return p.solo ? "accept_cluster_kernel (one workgroup per request, rows of the walked path only)"
                : "accept_cluster_kernel (cluster of workgroups per request, row slices held in LDS)";
}

void launch_accept(const AcceptArgs& a, hipStream_t stream) {
  if (a.B <= 0) return;
  const float c = kLog2e / a.temperature;
  const int n_t_rows = a.total_nodes + a.B;
  const int n_q_stat_rows = (a.q_kind == 0) ? a.n_q_rows : 0;
  const AcceptLayout lay = accept_layout(a.B, a.total_nodes, a.n_q_rows, a.V);
  unsigned char* ws = static_cast<unsigned char*>(a.workspace);
  const int n_cu = current_device_cus();
  {
    // bf16 logit rows (the default layout): one kernel that reads only the rows the walk reaches (it takes the
    // statistics of those rows itself; target statistics a caller supplies are not needed then)
    const bool vec0 = (a.V % 8 == 0) && aligned16(a.target) && aligned16(a.draft_q);
    const bool cluster_ok = vec0 && a.V >= 8 && a.V <= kClusterMaxV && a.t_dtype == kBF16 && a.q_dtype == kBF16 &&
                            a.q_kind == 0;
    if (cluster_ok && (a.path == 2 || (a.path == 0 && a.parent != nullptr && cluster_pays(a.B, a.V, n_cu)))) {
      const ClusterPlan plan = make_cluster_plan(a.B, a.V, a.max_nodes, a.parent != nullptr, n_cu, a.levels, a.slices);
      launch_accept_cluster(a, plan, a.patience >= 0 ? a.patience : 4000, ws + lay.msg_off, stream);
      return;
    }
  }
  SegStat* stats = reinterpret_cast<SegStat*>(ws);
  unsigned* words = reinterpret_cast<unsigned*>(ws + lay.words_off);      // start of the zeroed region
  if (progressive_stats(a)) {
    unsigned* node_cnt = reinterpret_cast<unsigned*>(ws + lay.prog_cnt_off);
    int* stop = reinterpret_cast<int*>(ws + lay.prog_stop_off);
    unsigned* arrived0 = reinterpret_cast<unsigned*>(ws + lay.arrived_off);
    const int n_cnt = a.total_nodes;
    hipLaunchKernelGGL(accept_prog_init_kernel, dim3((n_cnt + kStatThreads - 1) / kStatThreads), dim3(kStatThreads), 0, stream,
                       node_cnt, n_cnt, stop, arrived0, a.B);
    const int nseg = stats_segments(a.V);
    const dim3 grid_p(nseg, a.B, 2 * a.max_nodes + 1);
    const bool vec_p = (a.V % 8 == 0) && aligned16(a.target) && aligned16(a.draft_q);
    if (vec_p)
      hipLaunchKernelGGL(row_stats_prog_kernel<true>, grid_p, dim3(kStatThreads), 0, stream, a.target, a.t_dtype, n_t_rows,
                         a.draft_q, a.q_dtype, a.n_q_rows, a.V, c, nseg, stats, a.node_offsets, a.q_row, a.draft_tokens,
                         a.u_accept, node_cnt, stop, a.max_nodes);
    else
      hipLaunchKernelGGL(row_stats_prog_kernel<false>, grid_p, dim3(kStatThreads), 0, stream, a.target, a.t_dtype, n_t_rows,
                         a.draft_q, a.q_dtype, a.n_q_rows, a.V, c, nseg, stats, a.node_offsets, a.q_row, a.draft_tokens,
                         a.u_accept, node_cnt, stop, a.max_nodes);
  } else if (!a.target_stats_ready) {
    // rows nobody was drawn from exist only when there are more draft rows than nodes
    const bool sparse_q = n_q_stat_rows > a.total_nodes;
    launch_row_stats(a.target, a.t_dtype, n_t_rows, a.draft_q, a.q_dtype, n_q_stat_rows, a.V, c, stats, stream, words,
                     static_cast<int>(lay.n_zero_words), sparse_q ? a.q_row : nullptr, a.total_nodes);
  } else if (n_q_stat_rows > 0) {
    // the target rows' entries were written by the LM-head kernel; only the draft rows are left
    launch_row_stats(a.draft_q, a.q_dtype, n_q_stat_rows, nullptr, 0, 0, a.V, c,
                     stats + static_cast<size_t>(n_t_rows) * stats_segments(a.V), stream, words,
                     static_cast<int>(lay.n_zero_words));
  } else {
    hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(kStatThreads), 0, stream, words,
                       static_cast<int>(lay.n_zero_words));
  }
  AcceptParams P;
  P.B = a.B; P.V = a.V; P.n_t_rows = n_t_rows; P.n_q_rows = a.n_q_rows > 0 ? a.n_q_rows : 1; P.nseg = stats_segments(a.V);
  P.node_offsets = a.node_offsets; P.parent = a.parent; P.draft_tokens = a.draft_tokens;
  P.target = a.target; P.t_dtype = a.t_dtype;
  P.draft_q = a.draft_q; P.q_dtype = a.q_dtype; P.q_kind = a.q_kind;
  P.q_row = a.q_row; P.c = c; P.u_accept = a.u_accept; P.u_resample = a.u_resample;
  P.accept_len = a.accept_len; P.out_tokens = a.out_tokens; P.out_stride = a.out_stride;
  P.stop_node = a.stop_node; P.dbg_ratio = a.dbg_ratio; P.stats = stats;
  P.desc = reinterpret_cast<PassDesc*>(ws + lay.desc_off);
  P.part = reinterpret_cast<PartSlot*>(ws + lay.part_off);
  if (linear_path(a)) {
    const int unit_classes = linear_unit_classes(a.B, a.V, n_cu);
    const int U = (a.V + unit_classes - 1) / unit_classes;
    P.helpers = 0; P.patience = 0; P.parent = nullptr;
    double* partial = reinterpret_cast<double*>(ws + lay.lin_off);
    unsigned* arrived = reinterpret_cast<unsigned*>(ws + lay.arrived_off);
    const bool vec_l = (a.V % 8 == 0) && aligned16(a.target) && aligned16(a.draft_q);
    const dim3 grid_l(static_cast<unsigned>(a.B) * U);
    if (vec_l) hipLaunchKernelGGL((accept_linear_kernel<true>), grid_l, dim3(kLinThreads), 0, stream, P, partial, arrived, U, unit_classes);
    else hipLaunchKernelGGL((accept_linear_kernel<false>), grid_l, dim3(kLinThreads), 0, stream, P, partial, arrived, U, unit_classes);
    return;
  }
  // Helpers pay when a pass is long against a hand-off between compute units (a few microseconds):
  // vocabularies of 64k classes and more; masters plus helpers stay within one workgroup per compute unit.
  int helpers = 0;
  if (a.V >= 65536) {
    helpers = n_cu / a.B - 1;
    helpers = helpers < 0 ? 0 : (helpers > kMaxHelpers ? kMaxHelpers : helpers);
  }
  if (a.helpers >= 0 && a.helpers <= kMaxHelpers && a.B * (1 + a.helpers) <= n_cu) helpers = a.helpers;   // per-call tuning
  P.helpers = helpers;
  P.patience = (a.patience >= 0 && a.patience <= 1000000) ? a.patience : 400;   // default: a few hundred microseconds
  const dim3 grid(a.B * (1 + helpers));
  const bool vec = (a.V % 8 == 0) && aligned16(a.target) && aligned16(a.draft_q);
  const bool fast = vec && a.V >= 8 && a.t_dtype == kBF16 && a.q_dtype == kBF16 && a.q_kind == 0;
  if (fast) hipLaunchKernelGGL((accept_walk_kernel<true, true>), grid, dim3(kWalkThreads), 0, stream, P);
  else if (vec) hipLaunchKernelGGL((accept_walk_kernel<true, false>), grid, dim3(kWalkThreads), 0, stream, P);
  else hipLaunchKernelGGL((accept_walk_kernel<false, false>), grid, dim3(kWalkThreads), 0, stream, P);
}

}  // namespace specv
