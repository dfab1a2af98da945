// Acceptance-rejection walk of Section 2.1 (accept x when q(x) <= o(x), else reject with
// probability 1 - o(x)/q(x); replacement from norm(max(0, o - q)); bonus token when nothing is
// rejected; siblings of a draft tree by recursive rejection) for bf16 logit rows, as ONE kernel
// that reads only the rows the walk reaches.
//
// A request is walked by a cluster of C = LV x SL workgroups on different compute units.  The walk
// proceeds in windows: the current node and its chain of first children (LV levels, the speculated
// continuation of the walk).  Workgroup (lv, sl) loads vocabulary slice sl of the row pair of level
// lv (the node's target row and the draft row its children were drawn from) ONCE into its LDS,
// reduces its part of the softmax statistics, and all workgroups exchange their parts through small
// tagged messages in device memory.  Every workgroup then takes the same accept decisions from the
// same numbers (a replicated state machine: nothing has to be broadcast).  A rejection needs the
// mass of max(0, r - q): the workgroups of that level sum their slices FROM LDS and exchange
// again; the final inverse-CDF draw locates the slice from the exchanged sums and the workgroup that
// holds it finds the token in its LDS.  Rows behind the first rejection are never read, and no
// row is read twice.
//
// Messages.  One message = four 64-bit words {data : tag}, written with relaxed device-scope stores
// and read with relaxed device-scope loads; a word is valid when its tag equals the round number, so
// no ordering between words is needed.  Every workgroup posts in every round (a dummy when it has
// nothing to add) into one of two buffers chosen by the round's parity: a workgroup can post round
// r+2 only after it has seen every peer's round r+1, i.e. after every peer has finished reading
// round r, so two buffers suffice.  The buffers are zeroed by a small kernel launched ahead.
//
// No wait is unbounded and the result never depends on a peer making progress: a workgroup that does
// not see a round complete within its patience leaves; if it is the cluster's first workgroup (the
// owner, which writes the outputs) it marks its messages "abort" so the others leave too, and walks
// the request alone, computing every slice's part itself in the same order and with the same
// arithmetic (the results are bit-identical to the cluster's).  Clusters of one workgroup (large
// batches) work this way from the start.
#include "common.h"
#include "kernels.h"

namespace specv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kClThreads = 256;             // four waves, one per SIMD: the per-wave reductions and the replicated
                                            // scalar steps cost a quarter of what sixteen waves would pay
constexpr int kClWaves = kClThreads / kWave;
constexpr int kClUnit = kClThreads * 8;        // logits one workgroup-wide 16-byte load covers (2048)
constexpr int kClNodes = 128;
constexpr int kClMaxUpt = 16;                  // units per slice: 16 x 4 KiB per row, two rows = 128 KiB of LDS
constexpr int kClMaxParts = kClMaxUpt * kClWaves;
constexpr unsigned kClAbort = 0xffffffffu;
constexpr uint32_t kNegInf2 = 0xff80ff80u;     // two bf16 -inf

struct ClusterParams {
  int B, V, n_q_rows;
  const int32_t* node_offsets;
  const int32_t* parent;
  const int32_t* draft_tokens;
  const uint16_t* target;
  const uint16_t* draft_q;
  const int32_t* q_row;
  float c;                        // log2(e) / T
  const float* u_accept;
  const float* u_resample;
  int32_t* accept_len;
  int32_t* out_tokens; int out_stride;
  int32_t* stop_node;
  float* dbg_ratio;
  int LV, SL;                     // window levels x vocabulary slices = workgroups per request
  int UPT;                        // units (2048 logits) per slice
  int solo;                       // one workgroup per request, which computes all LV x SL parts itself
  int patience;                   // polls the owner spends on one round before it walks alone
  unsigned long long* msg;        // [B][2 buffers][C][2 messages][4 words]
};

template <typename T> __device__ __forceinline__ T cl_ld(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ void cl_st(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void cl_unpack(u32x4 r, float (&x)[8]) {
  x[0] = bf16_lo(r[0]); x[1] = bf16_hi(r[0]); x[2] = bf16_lo(r[1]); x[3] = bf16_hi(r[1]);
  x[4] = bf16_lo(r[2]); x[5] = bf16_hi(r[2]); x[6] = bf16_lo(r[3]); x[7] = bf16_hi(r[3]);
}

// Whole-wave reductions through the data-parallel-primitive path of the vector ALU (a few cycles per
// step, against a trip through the LDS crossbar per step for a shuffle): an inclusive scan inside
// each row of 16 lanes (row_shr 1, 2, 4, 8), then lane 15 of rows 0 and 2 is broadcast into rows 1 and 3
// (row_bcast:15) and lane 31 into rows 2 and 3 (row_bcast:31); lane 63 then holds the result, which
// is read back as a wave-uniform value.  Lanes without a source keep `old`, the identity.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xf, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xf, false);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_sum_dpp(double x) {
  x += dpp_f64<0x111, 0xf>(x);
  x += dpp_f64<0x112, 0xf>(x);
  x += dpp_f64<0x114, 0xf>(x);
  x += dpp_f64<0x118, 0xf>(x);
  x += dpp_f64<0x142, 0xa>(x);
  x += dpp_f64<0x143, 0xc>(x);
  const int lo = __builtin_amdgcn_readlane(__double2loint(x), 63);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(x), 63);
  return __hiloint2double(hi, lo);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max_step(float x) {
  const int ninf = 0xff800000;
  const int y = __builtin_amdgcn_update_dpp(ninf, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
  return fmaxf(x, __int_as_float(y));
}
__device__ __forceinline__ float wave_max_dpp(float x) {
  x = dpp_max_step<0x111, 0xf>(x);
  x = dpp_max_step<0x112, 0xf>(x);
  x = dpp_max_step<0x114, 0xf>(x);
  x = dpp_max_step<0x118, 0xf>(x);
  x = dpp_max_step<0x142, 0xa>(x);
  x = dpp_max_step<0x143, 0xc>(x);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// Statistics of one level of the window: row maxima and reciprocal sums of 2^((l - max) c).
struct LevelStats {
  float mp, mq;
  double izp, izq;
};

// Weights of eight consecutive classes at residual level L:
//   r_0 = p;  w_k = max(0, r_{k-1} - q);  r_k = w_k / R_k,  R_k = sum_v w_k(v);
// the weight of level L is w_L (unnormalised; p itself at level 0).  Classes beyond the vocabulary
// hold -inf logits and get weight 0.  Per-class values are fp32, sums over classes fp64.
__device__ __forceinline__ void cl_weights(u32x4 rp, u32x4 rq, const LevelStats& S, float c, int L,
                                           const float* __restrict__ inv_R, float (&w)[8]) {
  float lp[8], lq[8], q[8];
  cl_unpack(rp, lp);
  cl_unpack(rq, lq);
  const float izp = static_cast<float>(S.izp), izq = static_cast<float>(S.izq);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    w[j] = fast_exp2((lp[j] - S.mp) * c) * izp;
    q[j] = 0.f;
    if (L > 0) q[j] = fast_exp2((lq[j] - S.mq) * c) * izq;
  }
  for (int k = 0; k < L; ++k) {
    const float scale = (k + 1 < L) ? inv_R[k] : 1.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = fmaxf(w[j] - q[j], 0.f) * scale;
  }
}

__global__ __launch_bounds__(kClThreads) void accept_cluster_kernel(ClusterParams P) {
  // the slice this workgroup holds: [target row, draft row][UPT units][thread] x 16 bytes; a thread
  // only ever touches its own 16-byte slots, so no barrier orders these accesses
  extern __shared__ __align__(16) unsigned char cl_rows[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int SL = P.SL, LV = P.LV, C = SL * LV, UPT = P.UPT;
  const int CP = P.solo ? 1 : C;                  // workgroups that really exist per request
  const int b = blockIdx.x / CP, rank = blockIdx.x - b * CP;
  const int my_lv = rank / SL, my_sl = rank - my_lv * SL;
  const bool owner = rank == 0;
  const int V = P.V;
  const float c = P.c;

  __shared__ int sh_par[kClNodes], sh_tok[kClNodes], sh_qrow[kClNodes];
  __shared__ float sh_u[kClNodes], sh_lp[kClNodes], sh_lq[kClNodes];   // uniforms; raw logits of the drafted tokens
  __shared__ int sh_fc[kClNodes + 1];          // first child of node cur at [cur + 1], -2 = none
  __shared__ int sh_chain[16];                 // nodes of the window, -2 = the chain has ended
  __shared__ double sh_val[64];                // gathered messages
  __shared__ float sh_aux[64];
  __shared__ double sh_e[64];
  __shared__ float sh_M[2][16];                // per level: maximum of the target row / the draft row
  __shared__ double sh_iZ[2][16];              //            reciprocal sums
  __shared__ __align__(16) float sh_wm[2][kClWaves];
  __shared__ double sh_ws[2][kClWaves];        // per-wave sums of the slice held in LDS
  __shared__ double sh_part[kClMaxParts];      // its per-(unit, wave) sums (computed for the draw only)
  __shared__ double sh_invR[kClNodes];
  __shared__ float sh_invRf[kClNodes];
  __shared__ int sh_status;
  const int n_parts = UPT * kClWaves;          // <= 64

  const int o = P.node_offsets[b];
  int n = P.node_offsets[b + 1] - o;
  n = n < 0 ? 0 : (n > kClNodes ? kClNodes : n);
  const int64_t trow0 = static_cast<int64_t>(o) + b;
  const double u_res = static_cast<double>(P.u_resample[b]);

  // ---- the target row of this workgroup's level, when it is known before the node arrays arrive (the
  // root's row; any level of a linear draft): its loads go out first and overlap the dependent reads below
  const bool early_t = !P.solo && (my_lv == 0 || P.parent == nullptr) && my_lv - 1 < n;
  u32x4 early_r[kClMaxUpt];
  {
    const uint16_t* tp = P.target + (trow0 + my_lv) * static_cast<int64_t>(V);
    const u32x4 ninf = {kNegInf2, kNegInf2, kNegInf2, kNegInf2};
#pragma unroll
    for (int u = 0; u < kClMaxUpt; ++u) {
      const int e = (my_sl * UPT + u) * kClUnit + tid * 8;
      early_r[u] = ninf;
      if (early_t && u < UPT && e < V) early_r[u] = *reinterpret_cast<const u32x4*>(tp + e);
    }
  }

  // ---- node arrays (indices come from device memory the host cannot check: clamp them) ----
  if (tid < kClNodes) {
    int par = -2, tok = 0, qr = 0;
    float u = 0.f;
    if (tid < n) {
      par = P.parent ? P.parent[o + tid] : tid - 1;
      if (par < -1 || par >= tid) par = -1;
      tok = min(max(P.draft_tokens[o + tid], 0), V - 1);
      qr = min(max(P.q_row[o + tid], 0), P.n_q_rows - 1);
      u = P.u_accept[o + tid];
      if (owner && P.dbg_ratio) P.dbg_ratio[o + tid] = __builtin_nanf("");
    }
    sh_par[tid] = par; sh_tok[tid] = tok; sh_qrow[tid] = qr; sh_u[tid] = u;
    sh_invRf[tid] = 0.f;
    sh_invR[tid] = 0.0;
  }
  if (tid <= kClNodes) sh_fc[tid] = kClNodes;
  __syncthreads();
  if (tid < n) atomicMin(&sh_fc[sh_par[tid] + 1], tid);      // first child = lowest index among the children
  // the two logits of every drafted token, kept in registers until the first round's loads are out
  float g_lp = 0.f, g_lq = 0.f;
  if (tid < n) g_lp = bf16_bits_to_float(P.target[(trow0 + 1 + sh_par[tid]) * static_cast<int64_t>(V) + sh_tok[tid]]);
  __syncthreads();
  // the draft row of a sibling group is the one its first child names (the row the slices hold for that group)
  if (tid < n) {
    const int fc = min(sh_fc[sh_par[tid] + 1], kClNodes - 1);
    g_lq = bf16_bits_to_float(P.draft_q[static_cast<int64_t>(sh_qrow[fc]) * V + sh_tok[tid]]);
  }
  if (tid <= kClNodes && sh_fc[tid] >= kClNodes) sh_fc[tid] = -2;   // no child
  __syncthreads();
  // lane l looks after nodes l and l + 64; nodes that do not exist hold an impossible parent
  const int my_parent = (lane < n) ? sh_par[lane] : -3;
  const int my_parent_hi = (lane + 64 < n) ? sh_par[lane + 64] : -3;

  // ---- the slice held in LDS ----
  auto row_p = [&](int u) -> u32x4* { return reinterpret_cast<u32x4*>(cl_rows) + (u * kClThreads + tid); };
  auto row_q = [&](int u) -> u32x4* { return reinterpret_cast<u32x4*>(cl_rows) + ((UPT + u) * kClThreads + tid); };
  if (early_t) {
#pragma unroll
    for (int u = 0; u < kClMaxUpt; ++u)
      if (u < UPT) *row_p(u) = early_r[u];
  }
  // (a node < -1 stands for "the chain has ended"; skip_t: the target part is in LDS already)
  auto load_slice = [&](int node, int sl, bool skip_t = false) {
    const bool exists = node >= -1;
    node = max(node, -1);
    const int fcn = exists ? sh_fc[node + 1] : -2;
    const uint16_t* tp = P.target + (trow0 + 1 + node) * static_cast<int64_t>(V);
    const uint16_t* qp = P.draft_q + static_cast<int64_t>(sh_qrow[max(fcn, 0)]) * V;
    const u32x4 ninf = {kNegInf2, kNegInf2, kNegInf2, kNegInf2};
    u32x4 tp_r[kClMaxUpt], tq_r[kClMaxUpt];
#pragma unroll
    for (int u = 0; u < kClMaxUpt; ++u) {         // all loads first: up to 8 x 16 bytes in flight per thread
      const int e = (sl * UPT + u) * kClUnit + tid * 8;
      tp_r[u] = ninf;
      tq_r[u] = ninf;
      if (u < UPT && exists && e < V) {           // V is a multiple of 8: a chunk is inside or outside
        if (!skip_t) tp_r[u] = *reinterpret_cast<const u32x4*>(tp + e);
        if (fcn >= 0) tq_r[u] = *reinterpret_cast<const u32x4*>(qp + e);
      }
    }
#pragma unroll
    for (int u = 0; u < kClMaxUpt; ++u)
      if (u < UPT) {
        if (!skip_t) *row_p(u) = tp_r[u];
        *row_q(u) = tq_r[u];
      }
  };

  // Local statistics of the held slice: (max, sum 2^((l - max) c)) of the target part and the draft part.
  // The results are valid in wave 0 (the wave that posts them).
  auto slice_stats = [&](bool have_q, float& mp, double& zp, float& mq, double& zq) {
    float tp = -INFINITY, tq = -INFINITY;
    for (int u = 0; u < UPT; ++u) {
      float x[8];
      cl_unpack(*row_p(u), x);
#pragma unroll
      for (int j = 0; j < 8; ++j) tp = fmaxf(tp, x[j]);
      cl_unpack(*row_q(u), x);
#pragma unroll
      for (int j = 0; j < 8; ++j) tq = fmaxf(tq, x[j]);
    }
    tp = wave_max_dpp(tp);
    tq = wave_max_dpp(tq);
    __syncthreads();                              // earlier readers of sh_wm and sh_ws are done
    sh_wm[0][wave] = tp; sh_wm[1][wave] = tq;     // every lane of the wave stores the same value
    __syncthreads();
    mp = -INFINITY; mq = -INFINITY;
#pragma unroll
    for (int w = 0; w < kClWaves; w += 4) {
      const float4 a = *reinterpret_cast<const float4*>(&sh_wm[0][w]);
      const float4 b2 = *reinterpret_cast<const float4*>(&sh_wm[1][w]);
      mp = fmaxf(fmaxf(mp, fmaxf(a.x, a.y)), fmaxf(a.z, a.w));
      mq = fmaxf(fmaxf(mq, fmaxf(b2.x, b2.y)), fmaxf(b2.z, b2.w));
    }
    const float sp = (mp == -INFINITY) ? 0.f : mp, sq = (mq == -INFINITY) ? 0.f : mq;
    double ap = 0.0, aq = 0.0;
    for (int u = 0; u < UPT; ++u) {
      float x[8];
      cl_unpack(*row_p(u), x);
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += fast_exp2((x[j] - sp) * c);
      ap += static_cast<double>(sum);
      if (have_q) {
        cl_unpack(*row_q(u), x);
        sum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += fast_exp2((x[j] - sq) * c);
        aq += static_cast<double>(sum);
      }
    }
    ap = wave_sum_dpp(ap);
    aq = wave_sum_dpp(aq);
    sh_ws[0][wave] = ap; sh_ws[1][wave] = aq;
    __syncthreads();
    zp = wave_sum_dpp(lane < kClWaves ? sh_ws[0][lane] : 0.0);
    zq = wave_sum_dpp(lane < kClWaves ? sh_ws[1][lane] : 0.0);
  };

  // Sum of the level-L weights of the held slice (valid in every wave).
  auto slice_weight_sum = [&](const LevelStats& S, int L) -> double {
    double acc = 0.0;
    for (int u = 0; u < UPT; ++u) {
      float w[8];
      cl_weights(*row_p(u), *row_q(u), S, c, L, sh_invRf, w);
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += w[j];
      acc += static_cast<double>(sum);
    }
    acc = wave_sum_dpp(acc);
    __syncthreads();                              // earlier readers of sh_ws are done
    sh_ws[0][wave] = acc;
    __syncthreads();
    return wave_sum_dpp(lane < kClWaves ? sh_ws[0][lane] : 0.0);
  };

  // Per-(unit, wave) sums of the level-L weights of the held slice, in vocabulary order, for the draw.
  auto slice_parts = [&](const LevelStats& S, int L) {
    __syncthreads();
    for (int u = 0; u < UPT; ++u) {
      float w[8];
      cl_weights(*row_p(u), *row_q(u), S, c, L, sh_invRf, w);
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += w[j];
      const double d = wave_sum_dpp(static_cast<double>(sum));
      sh_part[u * kClWaves + wave] = d;
    }
    __syncthreads();
  };

  // ---- messages ----
  auto msg_ptr = [&](unsigned r, int wg, int k) {
    return P.msg + ((((static_cast<size_t>(b) * 2 + (r & 1u)) * C + wg) * 2 + k) * 4);
  };
  // every lane of wave 0 stores one of the four words (same values from the lanes that share a word)
  auto post = [&](unsigned r, int k, double val, float aux) {
    if (wave == 0) {
      const unsigned long long bits = static_cast<unsigned long long>(__double_as_longlong(val));
      const int w = lane & 3;
      const unsigned data = w == 0 ? static_cast<unsigned>(bits) : (w == 1 ? static_cast<unsigned>(bits >> 32)
                                   : (w == 2 ? __float_as_uint(aux) : 0u));
      cl_st(msg_ptr(r, rank, k) + w, (static_cast<unsigned long long>(data) << 32) | r);
    }
  };
  // 0: every peer's messages of round r are in sh_val / sh_aux; 1: gave up waiting; 2: the owner walks alone
  auto gather = [&](unsigned r, int nmsg) -> int {
    __syncthreads();                              // earlier readers of sh_val / sh_status are done
    if (wave == 0) {
      const int nslots = C * nmsg;
      const int my = min(lane, nslots - 1);       // lanes beyond repeat the last slot
      const unsigned long long* m = msg_ptr(r, my / nmsg, my % nmsg);
      const int limit = owner ? P.patience : 4 * P.patience + 16;
      int spins = 0, status = 0;
      unsigned long long w0 = 0, w1 = 0, w2 = 0;
      for (;;) {
        w0 = cl_ld(m); w1 = cl_ld(m + 1); w2 = cl_ld(m + 2);
        const bool ok = static_cast<unsigned>(w0) == r && static_cast<unsigned>(w1) == r && static_cast<unsigned>(w2) == r;
        const bool ab = static_cast<unsigned>(w0) == kClAbort;
        if (__any(ab)) { status = 2; break; }
        if (__all(ok)) break;
        if (++spins > limit) { status = 1; break; }
        __builtin_amdgcn_s_sleep(2);
      }
      if (status == 0) {
        sh_val[my] = __longlong_as_double(static_cast<long long>((w1 & 0xffffffff00000000ull) | (w0 >> 32)));
        sh_aux[my] = __uint_as_float(static_cast<unsigned>(w2 >> 32));
      }
      sh_status = status;
    }
    __syncthreads();
    return sh_status;
  };

  // ---- the walk; solo: this workgroup computes every slice's part itself ----
  auto walk = [&](const bool solo) -> int {
    int cur = -1, depth = 0;
    unsigned r = 0;
    int held_lv = -1, held_sl = -1;               // slice in registers (solo mode)
    for (int guard = 0; guard <= kClNodes + 1; ++guard) {
      // ---- window: the current node and its chain of first children ----
      __syncthreads();
      if (wave == 0) {                            // all lanes store the same words
        int cn = cur;
        for (int j = 0; j < LV; ++j) {
          sh_chain[j] = cn;
          cn = (cn >= -1) ? sh_fc[cn + 1] : -2;
        }
      }
      __syncthreads();
      ++r;
      if (!solo) {
        const int node = sh_chain[my_lv];
        float mp = -INFINITY, mq = -INFINITY;
        double zp = 0.0, zq = 0.0;
        load_slice(node, my_sl, guard == 0 && early_t);
        if (guard == 0 && tid < n) { sh_lp[tid] = g_lp; sh_lq[tid] = g_lq; }
        if (node >= -1) slice_stats(sh_fc[node + 1] >= 0, mp, zp, mq, zq);
        post(r, 0, zp, mp);
        post(r, 1, zq, mq);
        const int st = gather(r, 2);
        if (st) return st;
      } else {
        if (guard == 0 && tid < n) { sh_lp[tid] = g_lp; sh_lq[tid] = g_lq; }
        for (int v = 0; v < C; ++v) {
          const int lv = v / SL, sl = v - lv * SL;
          const int node = sh_chain[lv];
          float mp = -INFINITY, mq = -INFINITY;
          double zp = 0.0, zq = 0.0;
          if (node >= -1) {
            load_slice(node, sl);
            held_lv = lv; held_sl = sl;
            slice_stats(sh_fc[node + 1] >= 0, mp, zp, mq, zq);
          }
          __syncthreads();
          if (wave == 0) { sh_val[2 * v] = zp; sh_aux[2 * v] = mp; sh_val[2 * v + 1] = zq; sh_aux[2 * v + 1] = mq; }
        }
        __syncthreads();
      }
      // ---- merge the slices' parts per level: a wave per level, lane = (slice, row kind) ----
      for (int lvw = wave; lvw < LV; lvw += kClWaves) {
        const int sl = lane >> 1, kind = lane & 1;
        const bool have = sl < SL;
        const int idx = (lvw * SL + (have ? sl : 0)) * 2 + kind;
        const float m = have ? sh_aux[idx] : -INFINITY;
        const double z = have ? sh_val[idx] : 0.0;
        const float M0 = wave_max_dpp(kind == 0 ? m : -INFINITY);
        const float M1 = wave_max_dpp(kind == 1 ? m : -INFINITY);
        const float M = kind ? M1 : M0;
        const double e = (m == -INFINITY) ? 0.0 : z * exp2(static_cast<double>(m - M) * static_cast<double>(c));
        const double Z0 = wave_sum_dpp(kind == 0 ? e : 0.0);
        const double Z1 = wave_sum_dpp(kind == 1 ? e : 0.0);
        sh_M[0][lvw] = M0; sh_M[1][lvw] = M1;                   // every lane stores the same values
        sh_iZ[0][lvw] = 1.0 / Z0; sh_iZ[1][lvw] = 1.0 / Z1;
      }
      __syncthreads();

      // ---- decisions, level by level while the walk follows the chain ----
      int j = 0;
      bool new_window = false;
      while (!new_window) {
        LevelStats S;
        S.mp = sh_M[0][j]; S.izp = sh_iZ[0][j]; S.mq = sh_M[1][j]; S.izq = sh_iZ[1][j];
        int level = 0, sums_level = -1;
        double total = 0.0;

        // one exchange of level-L weight sums of pair j; the slices' sums land in sh_val[j*SL + sl]
        int fail = 0;
        auto sum_round = [&](int L) -> double {
          ++r;
          if (!solo) {
            double mine = 0.0;
            if (my_lv == j) mine = slice_weight_sum(S, L);
            post(r, 0, mine, 0.f);
            const int st = gather(r, 1);
            if (st) { fail = st; return 0.0; }
          } else {
            for (int sl = 0; sl < SL; ++sl) {
              if (held_lv != j || held_sl != sl) { load_slice(sh_chain[j], sl); held_lv = j; held_sl = sl; }
              const double t = slice_weight_sum(S, L);
              __syncthreads();
              if (wave == 0) sh_val[j * SL + sl] = t;
            }
            __syncthreads();
          }
          // total of the slices' sums (every wave of every workgroup: the same wave-level reduction)
          return wave_sum_dpp(lane < SL ? sh_val[j * SL + lane] : 0.0);
        };

        unsigned long long kids = __ballot(my_parent == cur && lane > cur);
        unsigned long long kids_hi = __ballot(my_parent_hi == cur && lane + 64 > cur);
        int accepted = -1;
        while (kids | kids_hi) {
          int ch;
          if (kids) { ch = __ffsll(static_cast<long long>(kids)) - 1; kids &= kids - 1; }
          else { ch = 64 + __ffsll(static_cast<long long>(kids_hi)) - 1; kids_hi &= kids_hi - 1; }
          const double qx = exp2((static_cast<double>(sh_lq[ch]) - static_cast<double>(S.mq)) * static_cast<double>(c)) * S.izq;
          double rx = exp2((static_cast<double>(sh_lp[ch]) - static_cast<double>(S.mp)) * static_cast<double>(c)) * S.izp;
          for (int k = 0; k < level; ++k) {
            double w = rx - qx;
            w = w > 0.0 ? w : 0.0;
            rx = w * sh_invR[k];
          }
          double ratio;
          if (qx > 0.0) ratio = rx / qx;
          else ratio = (rx > 0.0) ? INFINITY : 0.0;
          if (owner && P.dbg_ratio && wave == 0) P.dbg_ratio[o + ch] = static_cast<float>(ratio);
          if (static_cast<double>(sh_u[ch]) < ratio) { accepted = ch; break; }
          // rejected: mass of max(0, r - q)
          const double mass = sum_round(level + 1);
          if (fail) return fail;
          if (mass > 0.0) {
            __syncthreads();
            if (wave == 0) { sh_invR[level] = 1.0 / mass; sh_invRf[level] = static_cast<float>(1.0 / mass); }
            __syncthreads();
            ++level;
            sums_level = level;
            total = mass;
          } else {
            sums_level = -1;                       // the residual has no mass: r stays as it was
          }
        }
        if (accepted >= 0) {
          if (owner && wave == 0 && depth < P.out_stride)
            P.out_tokens[static_cast<int64_t>(b) * P.out_stride + depth] = sh_tok[accepted];
          ++depth;
          cur = accepted;
          if (j + 1 < LV && sh_chain[j + 1] == accepted) { ++j; continue; }   // its statistics are in this window
          new_window = true;
          continue;
        }

        // ---- no child, or every child rejected: draw from the level's weights by inverse CDF ----
        if (sums_level != level) {
          total = sum_round(level);
          if (fail) return fail;
        }
        const double target = u_res * total;
        // slice the crossing falls in: inclusive scan of the slices' sums over the lanes (SL <= 32)
        int s_hit;
        double before;
        {
          const double mine = lane < SL ? sh_val[j * SL + lane] : 0.0;
          double inc = mine;
#pragma unroll
          for (int d = 1; d < 32; d <<= 1) {
            const double tq = __shfl_up(inc, d, kWave);
            if (lane >= d) inc += tq;
          }
          unsigned long long hit = __ballot(lane < SL && inc > target);
          if (!hit) hit = __ballot(lane < SL && mine > 0.0) ? (1ull << (63 - __clzll(static_cast<long long>(__ballot(lane < SL && mine > 0.0))))) : 1ull;
          s_hit = __ffsll(static_cast<long long>(hit)) - 1;       // no crossing (rounding): the last slice with positive mass
          before = __shfl(inc - mine, s_hit, kWave);
        }
        if (solo && (held_lv != j || held_sl != s_hit)) {       // bring that slice back
          load_slice(sh_chain[j], s_hit);
          held_lv = j; held_sl = s_hit;
        }
        if (solo || (my_lv == j && my_sl == s_hit)) {
          slice_parts(S, level);
          // (unit, wave) part the crossing falls in: scan of the parts in vocabulary order (every wave alike)
          int p_hit;
          double run;
          {
            const double a = lane < n_parts ? sh_part[lane] : 0.0;
            double inc_a = a;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
              const double tq = __shfl_up(inc_a, d, kWave);
              if (lane >= d) inc_a += tq;
            }
            const unsigned long long hit_a = __ballot(lane < n_parts && before + inc_a > target);
            const unsigned long long pos_a = __ballot(lane < n_parts && a > 0.0);
            if (hit_a) p_hit = __ffsll(static_cast<long long>(hit_a)) - 1;
            else if (pos_a) p_hit = 63 - __clzll(static_cast<long long>(pos_a));      // rounding: last part with mass
            else p_hit = 0;
            run = before + __shfl(inc_a - a, p_hit, kWave);
          }
          const int u_hit = p_hit / kClWaves, w_hit = p_hit % kClWaves;
          if (wave == w_hit) {
            float w[8];
            cl_weights(*row_p(u_hit), *row_q(u_hit), S, c, level, sh_invRf, w);
            const int e0 = (s_hit * UPT + u_hit) * kClUnit + tid * 8;
            float lsf = 0.f;                       // summed exactly as the parts were
            int my_last = -1;
#pragma unroll
            for (int j2 = 0; j2 < 8; ++j2) { lsf += w[j2]; if (w[j2] > 0.f) my_last = e0 + j2; }
            const double ls = static_cast<double>(lsf);
            double inc = ls;                       // inclusive scan of the lane sums
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
              int tok = -1;
              double acc = run + inc - ls;
#pragma unroll
              for (int j2 = 0; j2 < 8; ++j2) {
                acc += static_cast<double>(w[j2]);
                if (tok < 0 && acc > target && w[j2] > 0.f) tok = e0 + j2;
              }
              if (tok < 0) tok = my_last;          // rounding inside the lane: its last positive class
              found = __shfl(tok, fl, kWave);
            }
            if (found < 0) {                       // rounding across lanes: last positive class of the part
              int ml = my_last;
#pragma unroll
              for (int d = 32; d > 0; d >>= 1) ml = max(ml, __shfl_xor(ml, d, kWave));
              found = ml >= 0 ? ml : min(V - 1, (s_hit * UPT + u_hit) * kClUnit + w_hit * 512);
            }
            if (depth < P.out_stride) P.out_tokens[static_cast<int64_t>(b) * P.out_stride + depth] = found;
          }
        }
        if (owner) {
          if (wave == 0) {
            P.accept_len[b] = depth;
            if (P.stop_node) P.stop_node[b] = cur;
          }
          for (int i = depth + 1 + tid; i < P.out_stride; i += kClThreads)
            P.out_tokens[static_cast<int64_t>(b) * P.out_stride + i] = -1;
        }
        return 0;
      }
    }
    return 0;
  };

  bool solo = P.solo != 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
    const int st = walk(solo);
    if (st == 0 || !owner) break;
    // the owner's peers are late or gone: tell them to leave and walk the request alone
    if (wave == 0)
      cl_st(P.msg + ((static_cast<size_t>(b) * 2 + ((lane >> 3) & 1)) * C * 2 + ((lane >> 2) & 1)) * 4 + (lane & 3),
            static_cast<unsigned long long>(kClAbort));
    __syncthreads();
    solo = true;
  }
}

__global__ __launch_bounds__(256) void cluster_zero_kernel(unsigned long long* __restrict__ words, int n) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) words[i] = 0ull;
}

ClusterPlan make_cluster_plan(int B, int V, int max_nodes, bool tree, int n_cu, int want_levels, int want_slices) {
  ClusterPlan p{};
  const int units = (V + kClUnit - 1) / kClUnit;
  if (n_cu > 1024) n_cu = 1024;
  int cmax = B > 0 ? n_cu / B : 1;
  cmax = cmax < 1 ? 1 : (cmax > 32 ? 32 : cmax);
  // levels worth speculating on: a linear draft can be accepted to its end; a tree's first-child
  // chain is followed with the probability that first children are accepted
  int lv_need = max_nodes + 1;
  const int lv_cap = tree ? 4 : 9;
  if (lv_need > lv_cap) lv_need = lv_cap;
  // The statistics of a slice are bound by the vector ALU of the one compute unit that holds it, so the
  // slices are made as small as the workgroups available allow; what is left over buys window levels.
  int best_upt = 0, best_lv = 0, best_sl = 0;
  for (int upt = 1; upt <= kClMaxUpt && best_upt == 0; upt *= 2) {
    const int sl = (units + upt - 1) / upt;
    if (upt < 4 && sl > 1 && want_slices <= 0) continue;      // rows are cut into slices of 8192 logits and more
    if (sl > cmax) continue;
    if (want_slices > 0 && sl != want_slices) continue;
    int lv = cmax / sl;
    if (lv > lv_need) lv = lv_need;
    if (want_levels > 0) { if (want_levels * sl > cmax || want_levels > 16) continue; lv = want_levels; }
    best_lv = lv; best_upt = upt; best_sl = sl;
  }
  if (best_upt != 0 && best_lv * best_sl == 1) p.solo = 1;       // a cluster of one exchanges nothing
  if (best_upt == 0) {
    // not even one slice set fits (or the batch exceeds the compute units): one workgroup per request,
    // which computes the parts of ceil(units / 16) slices in turn
    best_upt = kClMaxUpt;
    while (best_upt > 1 && units <= best_upt / 2) best_upt /= 2;
    if (want_slices > 0) {
      for (int upt = 1; upt <= kClMaxUpt; upt *= 2) if ((units + upt - 1) / upt == want_slices) best_upt = upt;
    }
    best_sl = (units + best_upt - 1) / best_upt;
    best_lv = 1;
    p.solo = 1;
  }
  p.upt = best_upt; p.levels = best_lv; p.slices = best_sl;
  return p;
}

size_t cluster_msg_bytes(int B) {
  // (workgroups of all clusters <= B + compute units <= B + 1024) x 2 buffers x 2 messages x 32 bytes
  return (static_cast<size_t>(B) + 1024) * 128;
}

void launch_accept_cluster(const AcceptArgs& a, const ClusterPlan& plan, int patience, void* msg, hipStream_t stream) {
  ClusterParams P;
  P.B = a.B; P.V = a.V; P.n_q_rows = a.n_q_rows > 0 ? a.n_q_rows : 1;
  P.node_offsets = a.node_offsets; P.parent = a.parent; P.draft_tokens = a.draft_tokens;
  P.target = static_cast<const uint16_t*>(a.target);
  P.draft_q = static_cast<const uint16_t*>(a.draft_q);
  P.q_row = a.q_row; P.c = kLog2e / a.temperature; P.u_accept = a.u_accept; P.u_resample = a.u_resample;
  P.accept_len = a.accept_len; P.out_tokens = a.out_tokens; P.out_stride = a.out_stride;
  P.stop_node = a.stop_node; P.dbg_ratio = a.dbg_ratio;
  P.LV = plan.solo ? 1 : plan.levels;
  P.SL = plan.slices;
  P.patience = patience;
  P.solo = plan.solo;
  P.UPT = plan.upt;
  P.msg = static_cast<unsigned long long*>(msg);
  const int C = plan.solo ? 1 : plan.levels * plan.slices;
  // a cluster of one workgroup exchanges nothing: SL stays the number of slices it computes in turn
  const dim3 grid(a.B * C);
  if (!plan.solo) {
    const int words = a.B * C * 16;
    hipLaunchKernelGGL(cluster_zero_kernel, dim3((words + 255) / 256 > 64 ? 64 : (words + 255) / 256), dim3(256), 0,
                       stream, P.msg, words);
  }
  const size_t lds = static_cast<size_t>(plan.upt) * 2 * kClThreads * 16;
  static std::atomic<uint64_t> attr_done{0};
  if (set_lds_once(&accept_cluster_kernel, static_cast<size_t>(kClMaxUpt) * 2 * kClThreads * 16, attr_done) != 0) return;
  hipLaunchKernelGGL(accept_cluster_kernel, grid, dim3(kClThreads), lds, stream, P);
}

}  // namespace specv
