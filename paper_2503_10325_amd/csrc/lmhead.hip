// LM-head projection fused with the first pass of the vocab-wide softmax: the matrix product the
// paper singles out as the bulk of verification on the target model (Section 3.1), producing the
// logits o_i of Section 2.1 as bf16 together with the per-(row, 8192-class segment) statistics
// (maximum, sum of 2^((l - max) c)) that the acceptance walk starts from, so that the logits are
// never read back for that purpose and never exist in fp32.
//
//   logits[r, v] = bf16( sum_k hidden[r, k] * weight[v, k] ),  fp32 accumulation on the matrix cores.
//
// Vocabulary-as-M tiling: A = 32 weight rows, B = 32 hidden rows, so both operands of
// v_mfma_f32_32x32x16_bf16 are 16 contiguous bytes per lane of a row-major operand and no
// transpose is needed anywhere.  One workgroup = 8 waves = 4 vocabulary tiles x 2 halves of the
// contraction, producing a [128 vocab x 128 rows] block; the two halves are added through LDS.
// With up to 128 rows (a verification batch) the weight matrix is read exactly once and the kernel
// is bound by that read.  More rows go to a second kernel (below) whose row blocks are scheduled
// next to each other on one XCD so that a weight tile is served by that XCD's L2.
//
// Both operands are staged global -> registers -> LDS in 64-wide slices of the contraction
// (rows padded to 144 bytes: conflict-free 16-byte operand reads), the weights three slices ahead,
// one barrier per slice.  Weight slices are private to their wave; hidden slices are shared by the four waves of a
// half.
#include <stdlib.h>

#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace specv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 lm_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float lm_f32x16;
typedef uint32_t lm_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t lm_u32x2 __attribute__((ext_vector_type(2)));

constexpr int kLmThreads = 512;
constexpr int kLmVB = 128;                          // vocabulary entries per workgroup (4 tiles of 32)
constexpr int kLmRB = 128;                          // hidden rows per workgroup (4 tiles of 32)
constexpr int kLmKC = 64;                           // contraction slice
constexpr int kLmPitch = kLmKC * 2 + 16;            // bytes per staged row
constexpr int kLmHidBuf = kLmRB * kLmPitch;         // one hidden slice
constexpr int kLmWBuf = 32 * kLmPitch;              // one weight slice of one wave
constexpr int kLmHidBytes = 2 * 2 * kLmHidBuf;      // 2 halves x 2 buffers
constexpr int kLmWBytes = 8 * 2 * kLmWBuf;          // 8 waves x 2 buffers
constexpr int kLmLds = kLmHidBytes + kLmWBytes;     // 147456 bytes
constexpr int kLmBlocksPerSeg = 8192 / kLmVB;       // block statistics per statistics segment
static_assert(4 * 64 * 64 * 4 <= kLmHidBytes, "split-K hand-over fits the hidden buffers");
static_assert(kLmBlocksPerSeg == 64, "one wave merges one segment");

struct LmParams {
  int rows, K, V;
  int nvb, nrb, total, per_xcd;
  int panel;               // wide kernel: vocabulary blocks per panel (0: row blocks of a vocabulary block adjacent)
  float c;
  const uint16_t* hidden;
  const uint16_t* weight;
  uint16_t* logits;
  float2* bstats;          // [rows][nvb]
};

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// Store the 32 vocabulary entries [vt, vt + 32) of one accumulator tile for this lane's row.  b[4 g + i] holds the
// lane's entry 8 g + 4 lh + i as bf16 bits.  full (uniform over the wave): the tile lies inside V, V is a multiple
// of 8 and the logits are 16-byte aligned; the two half-waves then exchange halves (lane ln ends up with all eight
// entries of group 2h, lane ln + 32 with those of group 2h + 1), so that every lane stores 16 bytes and one
// instruction writes 32 contiguous bytes per row - 8-byte stores left half of every 32-byte sector to a later
// instruction.
__device__ __forceinline__ void store_logit_tile(uint16_t* __restrict__ out_row, int vt, int lh, const uint32_t (&b)[16],
                                                 bool row_ok, bool full, int V) {
  if (full) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t w0x = b[8 * h + 0] | (b[8 * h + 1] << 16), w0y = b[8 * h + 2] | (b[8 * h + 3] << 16);
      const uint32_t w1x = b[8 * h + 4] | (b[8 * h + 5] << 16), w1y = b[8 * h + 6] | (b[8 * h + 7] << 16);
      const auto rx = __builtin_amdgcn_permlane32_swap(w0x, w1x, false, false);
      const auto ry = __builtin_amdgcn_permlane32_swap(w0y, w1y, false, false);
      lm_u32x4 v;
      v[0] = rx[0]; v[1] = ry[0]; v[2] = rx[1]; v[3] = ry[1];
      if (row_ok) *reinterpret_cast<lm_u32x4*>(out_row + vt + 8 * (2 * h + lh)) = v;
    }
  } else if (row_ok) {
    const bool vec4 = (V & 3) == 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int vg = vt + 8 * g + 4 * lh;
      if (vec4 && vg + 3 < V) {
        lm_u32x2 w;
        w.x = b[4 * g] | (b[4 * g + 1] << 16);
        w.y = b[4 * g + 2] | (b[4 * g + 3] << 16);
        *reinterpret_cast<lm_u32x2*>(out_row + vg) = w;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (vg + i < V) out_row[vg + i] = static_cast<uint16_t>(b[4 * g + i]);
      }
    }
  }
}

__global__ __launch_bounds__(kLmThreads) void lm_head_kernel(LmParams P) {
  extern __shared__ __align__(16) unsigned char lm_lds[];
  // consecutive logical blocks (the row blocks of one vocabulary block) on one XCD
  const int id = blockIdx.x;
  const int logical = (id & 7) * P.per_xcd + (id >> 3);
  if (logical >= P.total) return;
  const int rbk = logical % P.nrb, vb = logical / P.nrb;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mt = wave & 3, kh = wave >> 2;
  const int ln = lane & 31, lh = lane >> 5;
  unsigned char* hid = lm_lds + kh * 2 * kLmHidBuf;
  unsigned char* wst = lm_lds + kLmHidBytes + wave * 2 * kLmWBuf;
  const int K2 = P.K >> 1;
  const int nch = K2 / kLmKC;
  const int kbase = kh * K2;
  const int v0 = vb * kLmVB + mt * 32;
  const int r0 = rbk * kLmRB;

  // staging: 8 lanes cover the 128 bytes of one row slice
  const int t = tid & 255;
  const uint16_t* wsrc[4];
  const uint16_t* hsrc[4];
  int wdst[4], hdst[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int vrow = v0 + (lane >> 3) + 8 * j;
    vrow = vrow < P.V ? vrow : P.V - 1;
    wsrc[j] = P.weight + static_cast<int64_t>(vrow) * P.K + kbase + (lane & 7) * 8;
    wdst[j] = ((lane >> 3) + 8 * j) * kLmPitch + (lane & 7) * 16;
    int hrow = r0 + (t >> 3) + 32 * j;
    hrow = hrow < P.rows ? hrow : P.rows - 1;
    hsrc[j] = P.hidden + static_cast<int64_t>(hrow) * P.K + kbase + (t & 7) * 8;
    hdst[j] = ((t >> 3) + 32 * j) * kLmPitch + (t & 7) * 16;
  }
  // Weight slices (HBM) are fetched three slices ahead into a ring of two register sets (slice s in
  // set (s - 1) % 2); hidden slices (L2) one slice ahead.  Loads past the end repeat the last slice
  // and are never used: a branch around a load would make the wait counts after it pessimistic.
  lm_u32x4 wring[2][4], hreg[4];
  auto load_w = [&](int c, lm_u32x4 (&w)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = *reinterpret_cast<const lm_u32x4*>(wsrc[j] + c * kLmKC);
  };
  auto load_h = [&](int c) {
#pragma unroll
    for (int j = 0; j < 4; ++j) hreg[j] = *reinterpret_cast<const lm_u32x4*>(hsrc[j] + c * kLmKC);
  };
  auto store_slice = [&](int buf, const lm_u32x4 (&w)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      *reinterpret_cast<lm_u32x4*>(wst + buf * kLmWBuf + wdst[j]) = w[j];
      *reinterpret_cast<lm_u32x4*>(hid + buf * kLmHidBuf + hdst[j]) = hreg[j];
    }
  };

  lm_f32x16 acc[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;

  const int last = nch - 1;
  load_w(0, wring[0]);
  load_h(0);
  store_slice(0, wring[0]);
  load_w(1 < last ? 1 : last, wring[0]);
  load_w(2 < last ? 2 : last, wring[1]);
  load_h(1 < last ? 1 : last);
  __syncthreads();
  for (int c0 = 0; c0 < nch; c0 += 2) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int c = c0 + r;
      if (c < nch) {
        const int buf = c & 1;
        const unsigned char* wrd = wst + buf * kLmWBuf + ln * kLmPitch + lh * 16;
        const unsigned char* hrd = hid + buf * kLmHidBuf + ln * kLmPitch + lh * 16;
#pragma unroll
        for (int s = 0; s < kLmKC / 16; ++s) {
          const lm_bf16x8 a = __builtin_bit_cast(lm_bf16x8, *reinterpret_cast<const lm_u32x4*>(wrd + 32 * s));
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) {
            const lm_bf16x8 b =
                __builtin_bit_cast(lm_bf16x8, *reinterpret_cast<const lm_u32x4*>(hrd + nt * 32 * kLmPitch + 32 * s));
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[nt], 0, 0, 0);
          }
        }
        store_slice(buf ^ 1, wring[r]);                       // slice c + 1
        load_w(c + 3 < last ? c + 3 : last, wring[r]);
        load_h(c + 2 < last ? c + 2 : last);
        __syncthreads();
      }
    }
  }

  // add the two halves of the contraction: the upper half hands its tile over through LDS
  float* red = reinterpret_cast<float*>(lm_lds);
  if (kh == 1) {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[((mt * 64 + nt * 16 + r) << 6) + lane] = acc[nt][r];
  }
  __syncthreads();
  float2* sh_stat = reinterpret_cast<float2*>(lm_lds + kLmHidBytes);     // [4 tiles][128 rows]
  if (kh == 0) {
    const bool full = (P.V & 7) == 0 && v0 + 32 <= P.V && (reinterpret_cast<uintptr_t>(P.logits) & 15) == 0;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      const int row = r0 + nt * 32 + ln;
      const bool row_ok = row < P.rows;
      uint16_t* out = P.logits + static_cast<int64_t>(row_ok ? row : 0) * P.V;
      float x[16];
      uint32_t b[16];
      float m = -INFINITY;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int vg = v0 + 8 * g + 4 * lh;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = 4 * g + i;
          b[r] = f32_to_bf16_rne(acc[nt][r] + red[((mt * 64 + nt * 16 + r) << 6) + lane]);
          x[r] = (vg + i < P.V) ? __uint_as_float(b[r] << 16) : -INFINITY;
          m = fmaxf(m, x[r]);
        }
      }
      store_logit_tile(out, v0, lh, b, row_ok, full, P.V);
      const float mm = (m == -INFINITY) ? 0.f : m;
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) s += fast_exp2((x[r] - mm) * P.c);
      // the other half-wave holds the same row's other 16 classes
      const float mo = __shfl_xor(m, 32, kWave);
      const float so = __shfl_xor(s, 32, kWave);
      const float M = fmaxf(m, mo);
      const float MM = (M == -INFINITY) ? 0.f : M;
      const float mmo = (mo == -INFINITY) ? 0.f : mo;
      const float S = s * fast_exp2((mm - MM) * P.c) + so * fast_exp2((mmo - MM) * P.c);
      if (lh == 0) sh_stat[mt * kLmRB + nt * 32 + ln] = make_float2(M, S);
    }
  }
  __syncthreads();
  if (tid < kLmRB) {
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) M = fmaxf(M, sh_stat[i * kLmRB + tid].x);
    const float MM = (M == -INFINITY) ? 0.f : M;
    float S = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float2 st = sh_stat[i * kLmRB + tid];
      const float mi = (st.x == -INFINITY) ? 0.f : st.x;
      S += st.y * fast_exp2((mi - MM) * P.c);
    }
    const int row = r0 + tid;
    if (row < P.rows) P.bstats[static_cast<int64_t>(row) * P.nvb + vb] = make_float2(M, S);
  }
}

// ----------------------------------------------------------------------------------
// More than 128 rows: the product is bound by the matrix cores, and what limits them is operand
// delivery.  Each wave owns a [128 vocab x 64 rows] tile (8 accumulator tiles); the eight waves of a
// workgroup (two per SIMD, one workgroup per CU) share one 128-entry weight slice in LDS (each
// weight operand read feeds two matrix instructions) and cover 512 rows, so the slice is fetched and
// staged once per 512 rows.  The hidden operands never touch LDS: a small pre-pass re-lays
// the hidden states out in the order the matrix instruction reads them, so that one load
// instruction fetches 1 KB of contiguous memory (8 cache lines instead of 64 for a row-major
// operand, whose lanes walk down 32 different rows - the L1 tag rate, one line per clock, is what
// bounds such loads).  Inside a 64-wide slice the contraction index is permuted (lane half h, step
// j, element i  <->  k = 32 h + 8 j + i) in both operands alike.
//
// Packed hidden states: [row tile of 32][slice][step j = 0..3][lane 0..63] x 16 bytes,
// lane L holding hidden[32 tile + L % 32][64 slice + 32 (L / 32) + 8 j .. + 8]; rows past the end
// are zero.
//
// A last row block with few rows costs more than its rows: it needs one more pass over the weight
// matrix (from the memory-side cache at best), so the row count at which the product is cheapest per
// row is a multiple of 512.  Up to 32 remaining rows are handled by splitting the contraction over
// the waves of the workgroup (below); more than that keeps the ordinary path with some waves idle.
// ----------------------------------------------------------------------------------
constexpr int kLwThreads = 512;
constexpr int kLwRB = kLwThreads;                   // hidden rows per workgroup (64 per wave)
constexpr int kLwStage = kLmVB * 8 / kLwThreads;     // 16-byte loads per thread and weight slice (128 rows x 8)
constexpr int kLwStageRows = kLwThreads / 8;        // rows covered by one such load of the workgroup
static_assert(kLwStage * kLwStageRows == kLmVB && kLwStage * kLwThreads * 16 == kLmVB * kLmKC * 2, "staging covers one weight slice exactly");
constexpr int kLwLds = 8 * kLmHidBuf;               // two shared weight slices; a partial last row block: one per wave
static_assert(8 * 64 * 64 * 4 <= kLwLds, "the partial tiles of a split contraction fit");

__global__ __launch_bounds__(256) void lm_pack_hidden_kernel(const uint16_t* __restrict__ hidden, int rows, int K,
                                                             int64_t n_items, lm_u32x4* __restrict__ packed) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= n_items) return;
  const int nch = K / kLmKC;
  const int L = static_cast<int>(idx & 63);
  const int j = static_cast<int>((idx >> 6) & 3);
  const int64_t blk = idx >> 8;                      // tile * nch + slice
  const int c = static_cast<int>(blk % nch);
  const int64_t row = (blk / nch) * 32 + (L & 31);
  lm_u32x4 v = {0u, 0u, 0u, 0u};
  if (row < rows) v = *reinterpret_cast<const lm_u32x4*>(hidden + row * K + c * kLmKC + 32 * (L >> 5) + 8 * j);
  packed[idx] = v;
}

template <int PF2>
__global__ __launch_bounds__(kLwThreads) void lm_head_wide_kernel(LmParams P, const lm_u32x4* __restrict__ packed) {
  extern __shared__ __align__(16) unsigned char lm_lds[];
  const int id = blockIdx.x;
  int rbk, vb;
  if (P.panel > 0) {
    // vocabulary panels small enough for the memory-side cache: inside a panel all workgroups of row
    // block 0 come first, then row block 1 ... (consecutive ids spread over all XCDs), so that the
    // panel's weights are read from HBM once and by the later row blocks from that cache
    if (id >= P.total) return;
    const int per_panel = P.panel * P.nrb;
    const int pn = id / per_panel, rem = id - pn * per_panel;
    const int width = min(P.panel, P.nvb - pn * P.panel);
    rbk = rem / width;
    vb = pn * P.panel + rem - rbk * width;
  } else {
    const int logical = (id & 7) * P.per_xcd + (id >> 3);
    if (logical >= P.total) return;
    rbk = logical % P.nrb; vb = logical / P.nrb;
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int v0 = vb * kLmVB;
  const int r0 = rbk * kLwRB + wave * 64;             // this wave's first row
  const int left = P.rows - r0;
  // row tiles of this wave that hold rows; in a scalar register, so that the branches on it are scalar
  const int ntc = __builtin_amdgcn_readfirstlane(left >= 64 ? 2 : (left <= 0 ? 0 : (left + 31) >> 5));
  const int nch = P.K / kLmKC;

  // weight slice: 128 entries x 128 bytes, 8 lanes per row
  const uint16_t* wsrc[kLwStage];
  int wdst[kLwStage];
#pragma unroll
  for (int j = 0; j < kLwStage; ++j) {
    int vrow = v0 + (tid >> 3) + kLwStageRows * j;
    vrow = vrow < P.V ? vrow : P.V - 1;
    wsrc[j] = P.weight + static_cast<int64_t>(vrow) * P.K + (tid & 7) * 8;
    wdst[j] = ((tid >> 3) + kLwStageRows * j) * kLmPitch + (tid & 7) * 16;
  }
  // packed hidden operands of this wave's two row tiles (a wave without rows reads tile 0)
  const int tile0 = ntc > 0 ? (r0 >> 5) : 0;
  const lm_u32x4* hsrc[2];
  hsrc[0] = packed + static_cast<int64_t>(tile0) * nch * 256 + lane;
  hsrc[1] = packed + static_cast<int64_t>(ntc > 1 ? tile0 + 1 : tile0) * nch * 256 + lane;

  lm_f32x16 acc[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  // The whole slice loop exists three times - two, one or no row tile in this wave - and one scalar
  // branch picks the copy: branches inside the loop would split the accumulators' live ranges.
  // Every copy passes the same barriers.
  auto slice_loop = [&](auto n_tiles, auto ahead) {
    constexpr int NT = decltype(n_tiles)::value;
    // Weight slices are fetched PF slices ahead into a ring of PF - 1 register sets (8 registers per
    // set).  With up to 256 rows the product is bound by streaming the weights from HBM and two slices
    // ahead is a load latency short (kernel instance PF2 = 4); with more rows it is bound by the
    // matrix cores and the shorter ring measured faster (PF2 = 2).  Waves of a partial block have
    // little matrix work per slice to hide a load behind and always use the deep ring.  Hidden
    // operands: one set per HB slices ahead.
    constexpr int PF = decltype(ahead)::value;
    constexpr int R = PF - 1;
    constexpr int HB = NT == 2 ? 1 : R;
    lm_u32x4 wring[R][kLwStage];
    auto load_weight = [&](int c, lm_u32x4 (&w)[kLwStage]) {
#pragma unroll
      for (int j = 0; j < kLwStage; ++j) w[j] = *reinterpret_cast<const lm_u32x4*>(wsrc[j] + c * kLmKC);
    };
    auto store_weight = [&](int buf, const lm_u32x4 (&w)[kLwStage]) {
#pragma unroll
      for (int j = 0; j < kLwStage; ++j) *reinterpret_cast<lm_u32x4*>(lm_lds + buf * kLmHidBuf + wdst[j]) = w[j];
    };
    const int last = nch - 1;
    // Hidden operands: slice s lives in set s mod HB.  With two row tiles there is one set, reloaded
    // step by step with the next slice; with one tile there are three, so that this wave, which has
    // half the matrix work per slice, does not wait a load latency per slice either.
    lm_u32x4 b[HB][2][4];
    {
      lm_u32x4 w0[kLwStage];
      load_weight(0, w0);
      if constexpr (NT > 0) {
#pragma unroll
        for (int r = 0; r < HB; ++r) {
          const int cs = r < last ? r : last;
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int ni = 0; ni < NT; ++ni) b[r][ni][j] = hsrc[ni][(cs * 4 + j) * 64];
        }
      }
      store_weight(0, w0);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) load_weight(1 + r < last ? 1 + r : last, wring[r]);
    __syncthreads();
    // Loads and stores for the slices ahead are issued unconditionally (past the end they repeat the
    // last slice and are never used): a branch around a load would make every wait count after it
    // pessimistic.  The ring slot of a slice is static: R slices per trip.
    for (int c0 = 0; c0 < nch; c0 += R) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int c = c0 + r;
        if (c < nch) {
          const int buf = c & 1;
          const int cb = c + HB < last ? c + HB : last;
          const int cp = c + PF < last ? c + PF : last;
          if constexpr (NT > 0) {
            const unsigned char* wrd = lm_lds + buf * kLmHidBuf + ln * kLmPitch + lh * 64;
            // weight operands are read one step ahead; a step's hidden operands are dead after its
            // matrix instructions and are reloaded at once with those of HB slices later
            lm_u32x4 a[2][4];
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) a[0][mi] = *reinterpret_cast<const lm_u32x4*>(wrd + mi * 32 * kLmPitch);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              if (j < 3) {
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                  a[(j + 1) & 1][mi] = *reinterpret_cast<const lm_u32x4*>(wrd + mi * 32 * kLmPitch + 16 * (j + 1));
              }
#pragma unroll
              for (int mi = 0; mi < 4; ++mi) {
                acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(lm_bf16x8, a[j & 1][mi]),
                                                                     __builtin_bit_cast(lm_bf16x8, b[r % HB][0][j]), acc[mi][0], 0, 0, 0);
                if constexpr (NT > 1)
                  acc[mi][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(lm_bf16x8, a[j & 1][mi]),
                                                                       __builtin_bit_cast(lm_bf16x8, b[r % HB][1][j]), acc[mi][1], 0, 0, 0);
              }
#pragma unroll
              for (int ni = 0; ni < NT; ++ni) b[r % HB][ni][j] = hsrc[ni][(cb * 4 + j) * 64];
              __builtin_amdgcn_sched_barrier(0);
            }
          }
          store_weight(buf ^ 1, wring[r]);      // slice c + 1
          load_weight(cp, wring[r]);            // slice c + PF takes its place
          __syncthreads();
        }
      }
    }
  };
  // A row block of at most 32 rows (the remainder of rows / 512) would keep seven waves idle while
  // the workgroup crawls through its 64 slices one load latency at a time.  Instead the eight waves
  // split the contraction: wave w takes slices w, w + 8, ..., stages each in a weight buffer of its
  // own (no workgroup barrier in the loop) and accumulates the same row tile; the eight partial
  // tiles are then added through LDS into wave 0, which runs the ordinary epilogue.
  const bool tail_block = __builtin_amdgcn_readfirstlane(P.rows - rbk * kLwRB) <= 32;     // the same in every wave
  if (tail_block) {
    unsigned char* mine = lm_lds + wave * kLmHidBuf;
    const lm_u32x4* hs = packed + static_cast<int64_t>((rbk * kLwRB) >> 5) * nch * 256 + lane;
    const int wrow = lane >> 3, wseg = lane & 7;
    lm_u32x4 wl[16];
    auto issue = [&](int c) {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        int vrow = v0 + wrow + 8 * j;
        vrow = vrow < P.V ? vrow : P.V - 1;
        wl[j] = *reinterpret_cast<const lm_u32x4*>(P.weight + static_cast<int64_t>(vrow) * P.K + c * kLmKC + wseg * 8);
      }
    };
    // slices of this wave: wave, wave + 8, ...; a wave without slices (d_model < 512) loads slice 0 and
    // multiplies nothing.  (Two slices in flight per wave were no faster: what the remainder costs is
    // one more pass over the weights.)
    const int n_mine = wave < nch ? (nch - wave + 7) / 8 : 0;
    issue(wave < nch ? wave : 0);
    for (int i = 0; i < n_mine; ++i) {
      const int c = wave + 8 * i;
#pragma unroll
      for (int j = 0; j < 16; ++j)
        *reinterpret_cast<lm_u32x4*>(mine + (wrow + 8 * j) * kLmPitch + wseg * 16) = wl[j];
      lm_u32x4 b[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = hs[(c * 4 + j) * 64];
      issue(c + 8 < nch ? c + 8 : c);                   // unconditional: the last one repeats this slice
      const unsigned char* wrd = mine + ln * kLmPitch + lh * 64;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
          const lm_u32x4 a = *reinterpret_cast<const lm_u32x4*>(wrd + mi * 32 * kLmPitch + 16 * j);
          acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(lm_bf16x8, a),
                                                               __builtin_bit_cast(lm_bf16x8, b[j]), acc[mi][0], 0, 0, 0);
        }
      }
    }
    // add the eight partial tiles: 64 floats per lane and wave, 16 KB each
    __syncthreads();
    float* red = reinterpret_cast<float*>(lm_lds) + wave * (64 * 64);
    if (wave > 0) {
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[(mi * 16 + r) * 64 + lane] = acc[mi][0][r];
    }
    __syncthreads();
    if (wave == 0) {
      for (int w = 1; w < kLwThreads / 64; ++w) {
        const float* rw = reinterpret_cast<const float*>(lm_lds) + w * (64 * 64);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[mi][0][r] += rw[(mi * 16 + r) * 64 + lane];
      }
    } else {
      // the other waves hold partial sums of wave 0's rows, not tiles of their own
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mi][0][r] = 0.f;
    }
  } else {
    using Deep = std::integral_constant<int, 4>;
    if (ntc == 2) slice_loop(std::integral_constant<int, 2>{}, std::integral_constant<int, PF2>{});
    else if (ntc == 1) slice_loop(std::integral_constant<int, 1>{}, Deep{});
    else slice_loop(std::integral_constant<int, 0>{}, Deep{});
  }

  // each wave holds all 128 vocabulary entries of the block for its rows: statistics need no LDS
  const bool aligned = (P.V & 7) == 0 && (reinterpret_cast<uintptr_t>(P.logits) & 15) == 0;
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    const int row = r0 + ni * 32 + ln;
    const bool row_ok = row < P.rows;
    uint16_t* out = P.logits + static_cast<int64_t>(row_ok ? row : 0) * P.V;
    float m = -INFINITY;
    float x[4][16];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      uint32_t b[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int vg = v0 + 32 * mi + 8 * g + 4 * lh;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = 4 * g + i;
          b[r] = f32_to_bf16_rne(acc[mi][ni][r]);
          x[mi][r] = (vg + i < P.V) ? __uint_as_float(b[r] << 16) : -INFINITY;
          m = fmaxf(m, x[mi][r]);
        }
      }
      store_logit_tile(out, v0 + 32 * mi, lh, b, row_ok, aligned && v0 + 32 * mi + 32 <= P.V, P.V);
    }
    const float mm = (m == -INFINITY) ? 0.f : m;
    float s = 0.f;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += fast_exp2((x[mi][r] - mm) * P.c);
    const float mo = __shfl_xor(m, 32, kWave);
    const float so = __shfl_xor(s, 32, kWave);
    const float M = fmaxf(m, mo);
    const float MM = (M == -INFINITY) ? 0.f : M;
    const float mmo = (mo == -INFINITY) ? 0.f : mo;
    const float S = s * fast_exp2((mm - MM) * P.c) + so * fast_exp2((mmo - MM) * P.c);
    if (lh == 0 && row_ok) P.bstats[static_cast<int64_t>(row) * P.nvb + vb] = make_float2(M, S);
  }
}

// One wave per (row, 8192-class segment): the 64 block statistics of the segment become the entry
// the acceptance walk reads.
__global__ __launch_bounds__(kWave) void lm_stats_merge_kernel(const float2* __restrict__ bstats, int nvb, int nseg,
                                                               float c, SegStat* __restrict__ stats) {
  const int seg = blockIdx.x, row = blockIdx.y, lane = threadIdx.x;
  const int i = seg * kLmBlocksPerSeg + lane;
  float m = -INFINITY, s = 0.f;
  if (i < nvb) {
    const float2 b = bstats[static_cast<int64_t>(row) * nvb + i];
    m = b.x; s = b.y;
  }
  const float M = wave_max(m);
  const float MM = (M == -INFINITY) ? 0.f : M;
  const float mm = (m == -INFINITY) ? 0.f : m;
  const double z = wave_sum(static_cast<double>(s) * static_cast<double>(fast_exp2((mm - MM) * c)));
  if (lane == 0) {
    SegStat st;
    st.m = M; st.pad = 0.f; st.z = z;
    stats[static_cast<int64_t>(row) * nseg + seg] = st;
  }
}

// Workspace: [block statistics rows x ceil(V/128) x 8 bytes][packed hidden states, more than 128 rows only]
static size_t lm_bstats_bytes(int rows, int V) {
  const size_t nvb = (static_cast<size_t>(V) + kLmVB - 1) / kLmVB;
  return (static_cast<size_t>(rows) * nvb * sizeof(float2) + 255) / 256 * 256;
}

size_t lm_head_workspace_bytes(int rows, int d_model, int V) {
  size_t n = lm_bstats_bytes(rows, V) + 256;
  if (rows > kLmRB) n += static_cast<size_t>((rows + 31) / 32) * 32 * d_model * sizeof(uint16_t);
  return n;
}

size_t row_stats_bytes(int rows, int V) { return static_cast<size_t>(rows) * stats_segments(V) * sizeof(SegStat); }

int launch_lm_head(const LmHeadArgs& a, hipStream_t stream) {
  if (a.rows <= 0) return 0;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(lm_head_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kLmLds) != hipSuccess)
      return -1;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(lm_head_wide_kernel<2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLwLds) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(lm_head_wide_kernel<4>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLwLds) != hipSuccess)
      return -1;
    attr_set = true;
  }
  const bool wide = a.rows > kLmRB;
  LmParams P;
  P.rows = a.rows; P.K = a.d_model; P.V = a.V;
  P.nvb = (a.V + kLmVB - 1) / kLmVB;
  P.nrb = (a.rows + (wide ? kLwRB : kLmRB) - 1) / (wide ? kLwRB : kLmRB);
  P.total = P.nvb * P.nrb;
  P.per_xcd = (P.total + 7) / 8;
  // Several row blocks: panels of 128 vocabulary blocks (134 MB of weights at d_model = 4096), every
  // row block of a panel in turn, measured 5-10 % faster than keeping the row blocks of one
  // vocabulary block adjacent when the last row block is partial, and equal otherwise.
  P.panel = (wide && P.nrb > 1) ? 128 : 0;
#ifdef SPECV_DEV_KNOBS
  if (const char* e = getenv("SPECV_LM_PANEL")) {                       // sweeps only; normal builds read no environment
    const int v = atoi(e);
    if (v >= 0 && v <= 65536) P.panel = v;
  }
#endif
  P.c = kLog2e / a.temperature;
  P.hidden = static_cast<const uint16_t*>(a.hidden);
  P.weight = static_cast<const uint16_t*>(a.weight);
  P.logits = static_cast<uint16_t*>(a.logits);
  P.bstats = static_cast<float2*>(a.workspace);
  if (wide) {
    lm_u32x4* packed = reinterpret_cast<lm_u32x4*>(static_cast<unsigned char*>(a.workspace) + lm_bstats_bytes(a.rows, a.V));
    const int64_t n_items = static_cast<int64_t>((a.rows + 31) / 32) * (a.d_model / kLmKC) * 256;
    hipLaunchKernelGGL(lm_pack_hidden_kernel, dim3(static_cast<unsigned>((n_items + 255) / 256)), dim3(256), 0, stream,
                       P.hidden, a.rows, a.d_model, n_items, packed);
    if (a.rows <= 256)
      hipLaunchKernelGGL(lm_head_wide_kernel<4>, dim3(P.per_xcd * 8), dim3(kLwThreads), kLwLds, stream, P, packed);
    else
      hipLaunchKernelGGL(lm_head_wide_kernel<2>, dim3(P.per_xcd * 8), dim3(kLwThreads), kLwLds, stream, P, packed);
  } else {
    hipLaunchKernelGGL(lm_head_kernel, dim3(P.per_xcd * 8), dim3(kLmThreads), kLmLds, stream, P);
  }
  const int nseg = stats_segments(a.V);
  hipLaunchKernelGGL(lm_stats_merge_kernel, dim3(nseg, a.rows), dim3(kWave), 0, stream, P.bstats, P.nvb, nseg, P.c,
                     static_cast<SegStat*>(a.stats));
  return 0;
}

}  // namespace specv
