// Verify-attention for gfx950: the draft queries of each request attend over the paged
// bf16 KV cache (committed context + their draft ancestors), Section 2.1 / 4.2 of the
// paper (parallel verification with a tree-attention mask).
//
// Work decomposition.  All n*G query rows that share a KV head are processed together so every
// K/V byte is fetched once per KV head; long requests are cut into context chunks whose
// unnormalised partial results attn_combine_kernel merges (split-KV).  Two bodies:
//   token-split (stream_item, up to 64 rows per KV head, up to 128 in ragged batches): a 4-wave
//     workgroup per (request, KV head, chunk); every wave streams its own 32-token tiles (2 cache
//     pages): coalesced 16-byte global loads -> registers -> the wave's private LDS tile -> MFMA
//     operands; waves that share a 32-row query block merge through LDS.  Launched grid-mapped
//     (attn_stream_kernel) or, for small ragged batches, from a work list built on the device and
//     sorted by length (attn_stream_list_kernel).
//   row-split (rows_item; attn_rows_kernel, more rows, and inside the work list): the 4 or 8 waves of a
//     workgroup stage 64-token tiles together (double-buffered LDS; with 8 waves two tiles of global
//     loads in flight) and each owns one block of 32 query rows.  Instantiated a second time for
//     requests of 65 to 128 draft nodes (two ancestor-mask words per node).
// In both, S^T = K Q^T runs on v_mfma_f32_32x32x16_bf16 with the tokens as the M dimension, so
// each lane owns one query column and the online-softmax statistics need a single exchange
// between the half-waves.  V is transposed on its way into LDS (token pairs packed with v_perm).
// O^T = V^T P^T: the token-split body keeps bf16 operands (weights as a high and a low bf16 term);
// the row-split body converts V to fp16 while staging it and uses fp16 weights in one
// v_mfma_f32_32x32x16_f16 term.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"

namespace specv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = 4;
constexpr int kTile = 32;          // tokens per wave iteration
constexpr int kPage = 16;
// Head dimension of row m (0..31) of accumulator block db of O^T = V^T P^T: the V^T rows are stored by
// (d%8, d/8), see AttnCfg, and read in storage order.  With a = r >> 2, c = r & 3 of accumulator register r and
// the lane's half lh, m = 8a + 4lh + c; the registers (db, a) with equal (a % A, c), A = D/64, hold 8 consecutive
// head dimensions from acc_dim0<D>(a % A, c, lh) on, in the order j = (32*8/D) * db + a / A.
template <int D> __device__ __forceinline__ constexpr int acc_dim0(int am, int c, int lh) { return 8 * (8 * am + 4 * lh + c); }
constexpr int kMaxQ = 64;             // query nodes per request with one ancestor-mask word
constexpr int kMaxQWide = 128;        // ... with two (row-split kernels only)

template <int D>
struct AttnCfg {
  static constexpr int kCh = D / 8;                       // 16-byte chunks per token row
  static constexpr int kTokPerLoad = 64 / kCh;            // token rows one wave-wide load covers
  static constexpr int kLoads = kTile / kTokPerLoad;      // loads per tile per tensor (8 / 4)
  static constexpr int kKStride = D * 2 + 16;             // bytes; padded K row in LDS
  static constexpr int kKBytes = kTile * kKStride;
  static constexpr int kVStride = 80;                     // bytes; one V^T row = 32 tokens + pad
  // V^T row of head dimension d: sigma(d) = (d%8)*(D/8) + d/8.  Lane ln of the output product's block db reads
  // row 32*db + ln - consecutive rows, free of LDS bank conflicts at this stride (an odd multiple of 16 bytes) -
  // so accumulator row m of block db belongs to head dimension acc_dim<D>(db, m): see there.
  static constexpr int kVRows = D;
  static constexpr int kVBytes = kVRows * kVStride;
  static constexpr int kWaveLds = kKBytes + kVBytes;
  static constexpr int kQKSteps = D / 16;
  static constexpr int kDBlocks = D / 32;
  static constexpr int kPagesPerLoad = 16 / kCh;          // pages one round of V loads covers: 1 (D=128) / 2 (D=64)
  static constexpr int kVPageIters = 2 / kPagesPerLoad;
  static constexpr int kORedStride = D + 4;               // floats; padded row of the cross-wave reduction
};

struct AttnParams {
  const uint16_t* q;
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  const int32_t* block_table;
  const int32_t* ctx_len;
  const int32_t* q_offsets;
  const int32_t* parent;
  void* out;
  float* lse;
  float* ws_o;       // [rows, max_chunks, D] unnormalised partial outputs
  float2* ws_ml;     // [rows, max_chunks] (max in log2 units, sum)
  int B, Hq, Hkv, G, max_pages, chunk_tokens, max_chunks;
  int tau;           // > 0: a request is cut so that one wave streams at most tau tiles per work item
  int list_rows_min; // > 0 (work list only): requests with this many query rows per KV head use the row-split body
  int list_rows_units;
  int xcd_swizzle;            // grid-mapped row-split launch: consecutive workgroups of the logical order share an XCD
  int n_cap;                  // query nodes per request the launched kernels handle (64, or 128 with two mask words)  // eighths of a work-list unit that 32 tokens of such a request cost
  float c;           // scale * log2(e)
  int out_f32;
};

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The value held by the same lane of the other half-wave (lane ^ 32), through the gfx950 half-wave
// swap instead of an LDS round trip: after swapping the upper half of one copy with the lower half
// of another, lane l of the first copy holds x[l % 32] and of the second x[32 + l % 32].
__device__ __forceinline__ void half_pair(float x, float& lo_half, float& hi_half) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  lo_half = __uint_as_float(r[0]);
  hi_half = __uint_as_float(r[1]);
}
__device__ __forceinline__ float half_max(float x) {
  float a, b;
  half_pair(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float half_sum(float x) {
  float a, b;
  half_pair(x, a, b);
  return a + b;
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ u32x4 zero4() {
  u32x4 z = {0u, 0u, 0u, 0u};
  return z;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// Two fp32 values as two fp16 in one word (round toward zero: never rounds a finite value to infinity).
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
// A word of two bf16 values as two fp16 values.  Exact for magnitudes in [2^-14, 65504] (bf16 carries 8
// significant bits, fp16 11); smaller magnitudes land on the fp16 subnormal grid (absolute error < 2^-24),
// larger ones saturate at 65504.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) { return pack_f16(bf16_lo(w), bf16_hi(w)); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2 x = {static_cast<__bf16>(lo), static_cast<__bf16>(hi)};
  return __builtin_bit_cast(uint32_t, x);
}

// Waves of a token-split workgroup that share one query block, for R <= 128 query rows.
// A zero the compiler cannot see through.  Added to the thread id at the top of a work item's body, it ties the
// per-lane constants of that body (lane offsets, LDS addresses) to the item: in a kernel that loops over items
// of two different bodies they would otherwise be hoisted out of the loop and held in registers across both.
__device__ __forceinline__ int opaque_zero() {
  int z = 0;
  asm volatile("" : "+s"(z));
  return z;
}

__device__ __forceinline__ int stream_nslice(int R) {
  const int nqb = min(4, (R + 31) / 32);
  return nqb <= 1 ? 4 : (nqb <= 2 ? 2 : 1);
}

// Number of context chunks of a request with L tokens and n draft nodes.  The token-split,
// sorted-work-list launch (tau > 0) cuts by the number of tiles one wave streams; the other
// launches cut by tokens.  The attention kernels and the combine kernel all use this function.
// Work-list launches run requests with at least P.list_rows_min query rows per KV head through the row-split
// body (its waves share every staged tile; the token-split body stages a tile once per 32-row block).
__device__ __forceinline__ bool list_uses_rows(const AttnParams& P, int n) {
  return P.list_rows_min > 0 && n * P.G >= P.list_rows_min;
}

// Length of a request in the work list's unit, the 32-token tiles one wave of the token-split body streams.
// For the row-split body 32 tokens count P.list_rows_units eighths of a unit: batches of equal requests
// measure 5/8 (a 64-token tile takes 1.25 times a 32-token one), ragged batches of both kinds run best
// with 3/8 (seven seeds of the serving mix: 1 to 8 % ahead of 4/8); the host passes 3.
__device__ __forceinline__ int request_units(const AttnParams& P, int L, int n) {
  const int tiles = (L + kTile - 1) / kTile;
  if (list_uses_rows(P, n)) return (tiles * P.list_rows_units + 7) / 8;
  const int nslice = stream_nslice(min(n * P.G, 128));
  return (tiles + nslice - 1) / nslice;
}

__device__ __forceinline__ int request_chunks(const AttnParams& P, int L, int n) {
  if (P.tau > 0) return min(max(1, (request_units(P, L, n) + P.tau - 1) / P.tau), P.max_chunks);
  return max(1, (L + P.chunk_tokens - 1) / P.chunk_tokens);
}

// Token-split kernel (up to 128 query rows per KV head and workgroup).  The 4 waves of a
// workgroup take roles from the number of 32-row query blocks nqb of the request:
//   nqb = 1: the four waves stream every 4th tile for the same query block;
//   nqb = 2: two waves per query block, each streaming every 2nd tile;
//   nqb = 3, 4: one wave per query block, streaming every tile.
// Waves that share tokens fetch them separately (the repeats hit in L2: HBM traffic stays 1x).
// One work item: (request b, KV head kvh, context chunk, row group rg).  Every return below is
// workgroup-uniform.
template <int D>
__device__ __forceinline__ void stream_item(const AttnParams& P, unsigned char* smem, int b, int kvh, int chunk, int rg,
                                            int q0, int n, int ctx) {
  using C = AttnCfg<D>;
  const int tid = static_cast<int>(threadIdx.x) + opaque_zero(), lane = tid & 63, wave = tid >> 6;
  __builtin_assume(tid >= 0 && tid < kAttnThreads);
  const int ln = lane & 31, lh = lane >> 5;

  // (q0, n, ctx: first query row, number of query nodes (already capped at kMaxQ) and context length of request b)
  if (n <= 0) return;
  const int L = ctx + n;
  const int R = n * P.G;
  const int row0 = rg * 128;
  if (row0 >= R) return;
  const int nqb = min(4, (R - row0 + 31) / 32);             // query blocks of this workgroup
  const int nqbp = nqb <= 1 ? 1 : (nqb <= 2 ? 2 : 4);       // ... rounded up to a power of two
  const int nslice = kAttnWaves / nqbp;                     // waves sharing one query block
  const int my_qb = wave % nqbp, my_slice = wave / nqbp;
  const bool wave_active = my_qb < nqb;                     // wave-uniform
  const int nchunks = request_chunks(P, L, n);
  if (chunk >= nchunks) return;
  const int cb = (((L + nchunks - 1) / nchunks) + kTile - 1) & ~(kTile - 1);
  const int t_begin = chunk * cb;
  const int t_end = min(L, t_begin + cb);
  const int ntiles = (t_end - t_begin + kTile - 1) / kTile;

  unsigned char* tile_lds = smem + wave * C::kWaveLds;
  unsigned char* k_lds = tile_lds;
  unsigned char* v_lds = tile_lds + C::kKBytes;
  // Small arrays alias the tile memory: the ancestor masks are consumed before the first
  // tile is staged, the merge statistics live behind the cross-wave reduction buffer.
  unsigned long long* sh_anc = reinterpret_cast<unsigned long long*>(smem);            // [64]
  int* sh_par = reinterpret_cast<int*>(smem + 512);                                    // [64]
  float* sh_m = reinterpret_cast<float*>(smem + kAttnWaves * 32 * C::kORedStride * sizeof(float));  // [4][32]
  float* sh_l = sh_m + kAttnWaves * 32;                                                // [4][32]

  // ---- ancestor-or-self masks of the draft nodes (only chunks that reach the drafts) ----
  const bool touches_drafts = t_end > ctx;
  if (touches_drafts) {
    if (P.parent) {
      if (tid < kMaxQ) sh_par[tid] = (tid < n) ? P.parent[q0 + tid] : -1;
      __syncthreads();
    }
    if (tid < kMaxQ) {
      unsigned long long mask = 0;
      if (tid < n) {
        if (P.parent) {
          int a = tid;
          for (int g = 0; g <= tid && a >= 0; ++g) {
            mask |= 1ull << a;
            const int p = sh_par[a];
            a = (p >= a || p < -1) ? -1 : p;
          }
        } else {
          mask = (2ull << tid) - 1ull;
        }
      }
      sh_anc[tid] = mask;
    }
    __syncthreads();
  }

  // ---- this lane's query column ----
  const int row = row0 + 32 * my_qb + ln;
  const bool valid = row < R;
  const int node = valid ? row / P.G : 0;
  const int gq = valid ? row % P.G : 0;
  const unsigned long long my_anc = (touches_drafts && valid) ? sh_anc[node] : 0ull;
  bf16x8 qf[C::kQKSteps];
  {
    const uint16_t* qp = P.q + (static_cast<int64_t>(q0 + node) * P.Hq + kvh * P.G + gq) * D + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < C::kQKSteps; ++ks) {
      u32x4 v = zero4();
      if (valid) v = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
      qf[ks] = as_bf16x8(v);
    }
  }
  if (touches_drafts) __syncthreads();       // masks are in registers; the memory becomes tile space

  float m_run = -INFINITY, l_run = 0.f;
  f32x16 oacc[C::kDBlocks];
#pragma unroll
  for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;

  // ---- lane roles for the loads ----
  const int kc = lane % C::kCh;              // 16-byte chunk within the token row
  const int kt = lane / C::kCh;              // token row within one load instruction
  // V: each lane loads 4 consecutive tokens (4*va + i) of a page so that the transposed
  // LDS write packs them into 8 bytes.
  const int vgrp = lane / C::kCh;
  const int vg4 = vgrp & 3;
  const int va = ((vg4 & 1) << 1) | (vg4 >> 1);     // token group within the page
  const int vs_lane = vgrp >> 2;                     // page within one load (D=64 only)
  const int vhh = va & 1, vpart = va >> 1;

  const int32_t* bt = P.block_table + static_cast<int64_t>(b) * P.max_pages;
  const int64_t page_elems = static_cast<int64_t>(P.Hkv) * kPage * D;
  const int64_t head_off = static_cast<int64_t>(kvh) * kPage * D;

  u32x4 kr[C::kLoads], vr[C::kLoads];

  // Page ids are fetched one tile ahead of the K/V loads that need them, so the tile loads never
  // wait on a dependent block-table read.  They are wave-uniform: the loads below take the page
  // base from scalar registers and add a per-lane byte offset that never changes, so a tile costs
  // no address arithmetic and no branch.  Ids past the request's last page repeat the last page and
  // negative ids read page 0: the data is in bounds, and tokens at or beyond L are masked (K) or
  // zeroed before they reach LDS (V).
  const int last_page = (L - 1) / kPage;
  int pg[2] = {0, 0};
  auto fetch_pages = [&](int t) {
    if (t < ntiles) {
      const int lp = (t_begin + kTile * t) / kPage;
      pg[0] = bt[lp];
      pg[1] = bt[min(lp + 1, last_page)];
    }
  };
  const unsigned k_lane_off = static_cast<unsigned>(kt * D + kc * 8) * 2u;            // bytes
  const unsigned v_lane_off = static_cast<unsigned>(4 * va * D + kc * 8) * 2u;
  const int64_t page_bytes = page_elems * 2, head_bytes = head_off * 2;
  auto issue_loads = [&](int t) {
    const int p0 = max(__builtin_amdgcn_readfirstlane(pg[0]), 0);
    const int p1 = max(__builtin_amdgcn_readfirstlane(pg[1]), 0);
    const int64_t o0 = p0 * page_bytes + head_bytes, o1 = p1 * page_bytes + head_bytes;
    const unsigned char* kb[2] = {reinterpret_cast<const unsigned char*>(P.k_pool) + o0,
                                  reinterpret_cast<const unsigned char*>(P.k_pool) + o1};
    const unsigned char* vb[2] = {reinterpret_cast<const unsigned char*>(P.v_pool) + o0,
                                  reinterpret_cast<const unsigned char*>(P.v_pool) + o1};
#pragma unroll
    for (int j = 0; j < C::kLoads; ++j) {
      constexpr int kRowBytes = D * 2;
      const int tk0 = j * C::kTokPerLoad;                 // first token row of this load (compile time)
      kr[j] = *reinterpret_cast<const u32x4*>(kb[tk0 / kPage] + k_lane_off + (tk0 % kPage) * kRowBytes);
    }
#pragma unroll
    for (int pi = 0; pi < C::kVPageIters; ++pi) {
      // D = 128: one page per round (scalar base); D = 64: the two half-waves read the tile's two pages
      const unsigned char* base = (C::kPagesPerLoad == 2) ? (vs_lane ? vb[1] : vb[0]) : vb[pi];
#pragma unroll
      for (int i = 0; i < 4; ++i) vr[pi * 4 + i] = *reinterpret_cast<const u32x4*>(base + v_lane_off + i * D * 2);
    }
  };

  int t = my_slice;
  if (wave_active && t < ntiles) {
    fetch_pages(t);
    issue_loads(t);
    fetch_pages(t + nslice);
  }
  for (; wave_active && t < ntiles; t += nslice) {
    // ---- registers -> LDS ----
#pragma unroll
    for (int j = 0; j < C::kLoads; ++j) {
      const int tk = j * C::kTokPerLoad + kt;
      *reinterpret_cast<u32x4*>(k_lds + tk * C::kKStride + kc * 16) = kr[j];
    }
    const int tok0 = t_begin + kTile * t;
    if (tok0 + kTile > L) {                  // last, partial tile: stale cache slots must not reach O
#pragma unroll
      for (int pi = 0; pi < C::kVPageIters; ++pi)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = tok0 + kPage * (pi * C::kPagesPerLoad + vs_lane) + 4 * va + i;
          if (tok >= L) vr[pi * 4 + i] = zero4();
        }
    }
#pragma unroll
    for (int pi = 0; pi < C::kVPageIters; ++pi) {
      const int s = pi * C::kPagesPerLoad + vs_lane;
      const u32x4 w0 = vr[pi * 4 + 0], w1 = vr[pi * 4 + 1], w2 = vr[pi * 4 + 2], w3 = vr[pi * 4 + 3];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const uint32_t sel = half ? 0x07060302u : 0x05040100u;
          uint2 o;
          o.x = __builtin_amdgcn_perm(w1[k], w0[k], sel);    // tokens 4va, 4va+1 at dim 8kc+2k+half
          o.y = __builtin_amdgcn_perm(w3[k], w2[k], sel);    // tokens 4va+2, 4va+3
          const int vrow = (2 * k + half) * (D / 8) + kc;
          *reinterpret_cast<uint2*>(v_lds + vrow * C::kVStride + 32 * s + 16 * vhh + 8 * vpart) = o;
        }
      }
    }
    if (t + nslice < ntiles) {
      issue_loads(t + nslice);
      fetch_pages(t + 2 * nslice);
    }
    wave_lds_fence();

    // ---- S^T = K Q^T ----
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::kQKSteps; ++ks) {
      const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(k_lds + ln * C::kKStride + 32 * ks + 16 * lh));
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc, 0, 0, 0);
    }

    // ---- mask, online softmax ----
    const bool need_mask = tok0 + kTile > ctx;
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = sacc[r];
      if (need_mask) {
        const int pos = tok0 + 8 * (r >> 2) + 4 * lh + (r & 3);
        // branch-free on purpose: bitwise ops, no short-circuit control flow around the accumulator
          const bool ok = (pos < ctx) | ((pos < L) & (((my_anc >> ((pos - ctx) & 63)) & 1ull) != 0ull));
        v = ok ? v : -INFINITY;
        sacc[r] = v;
      }
      tmax = fmaxf(tmax, v);
    }
    tmax *= P.c;                                   // c > 0: the maximum commutes with the scaling
    tmax = half_max(tmax);
    const float m_new = fmaxf(m_run, tmax);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_safe);
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    // ---- P^T as two bf16 terms (value + rounding residual), 16 tokens at a time; O^T += V^T P^T ----
    // A single bf16 rounding of P (2^-9 relative) would dominate the output error; carrying the
    // rounding residual in a second bf16 term keeps ~16 bits of every weight.
    float psum = 0.f;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      u32x4 hi, lo;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float p0 = fast_exp2(fmaf(sacc[8 * s + 2 * j], P.c, -m_safe));
        const float p1 = fast_exp2(fmaf(sacc[8 * s + 2 * j + 1], P.c, -m_safe));
        psum += p0 + p1;
        const uint32_t h = pack_bf16(p0, p1);
        hi[j] = h;
        lo[j] = pack_bf16(p0 - bf16_lo(h), p1 - bf16_hi(h));
      }
      const bf16x8 phi = __builtin_bit_cast(bf16x8, hi), plo = __builtin_bit_cast(bf16x8, lo);
#pragma unroll
      for (int db = 0; db < C::kDBlocks; ++db) {
        const int vrow = 32 * db + ln;           // storage order: head dimension acc_dim of this lane
        const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(v_lds + vrow * C::kVStride + 32 * s + 16 * lh));
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, phi, oacc[db], 0, 0, 0);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, plo, oacc[db], 0, 0, 0);
      }
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    wave_lds_fence();
  }

  // ---- merge the waves that share a query block ----
  l_run = half_sum(l_run);
  __syncthreads();                         // every wave is done with its tile memory
  if (lane < 32) {
    sh_m[wave * 32 + lane] = m_run;
    sh_l[wave * 32 + lane] = l_run;
  }
  __syncthreads();
  float M = -INFINITY;
  for (int s = 0; s < nslice; ++s) M = fmaxf(M, sh_m[(my_qb + nqbp * s) * 32 + ln]);
  const float fscale = (m_run == -INFINITY) ? 0.f : fast_exp2(m_run - M);

  float* sh_o = reinterpret_cast<float*>(smem);        // [4 waves][32][kORedStride]
  if (wave_active) {
    constexpr int kA = D / 64, kQ = 256 / D;     // see acc_dim0
#pragma unroll
    for (int am = 0; am < kA; ++am)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = oacc[j / kQ][4 * ((j % kQ) * kA + am) + c] * fscale;
        float* dst = sh_o + (wave * 32 + ln) * C::kORedStride + acc_dim0<D>(am, c, lh);
        *reinterpret_cast<float4*>(dst) = make_float4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<float4*>(dst + 4) = make_float4(x[4], x[5], x[6], x[7]);
      }
  }
  __syncthreads();
  const int rn = tid >> 3;                               // query column this thread finalises
  const int rd0 = (tid & 7) * (D / 8);                   // first of its D/8 dims
  for (int qb = 0; qb < nqb; ++qb) {
    const int orow = row0 + 32 * qb + rn;
    if (orow >= R) continue;
    float Mq = -INFINITY;
    for (int s = 0; s < nslice; ++s) Mq = fmaxf(Mq, sh_m[(qb + nqbp * s) * 32 + rn]);
    float Ls = 0.f;
    float acc[D / 8];
#pragma unroll
    for (int i = 0; i < D / 8; ++i) acc[i] = 0.f;
    for (int s = 0; s < nslice; ++s) {
      const int w = qb + nqbp * s;
      const float mw = sh_m[w * 32 + rn];
      if (mw != -INFINITY) Ls += sh_l[w * 32 + rn] * fast_exp2(mw - Mq);
#pragma unroll
      for (int i = 0; i < D / 8; i += 4) {
        const float4 v = *reinterpret_cast<const float4*>(sh_o + (w * 32 + rn) * C::kORedStride + rd0 + i);
        acc[i] += v.x; acc[i + 1] += v.y; acc[i + 2] += v.z; acc[i + 3] += v.w;
      }
    }
    const int onode = orow / P.G, og = orow % P.G;
    const int64_t grow = static_cast<int64_t>(q0 + onode) * P.Hq + kvh * P.G + og;
    if (nchunks == 1) {
      const float inv = 1.f / Ls;
      if (P.out_f32) {
        float* o = static_cast<float*>(P.out) + grow * D + rd0;
#pragma unroll
        for (int i = 0; i < D / 8; ++i) o[i] = acc[i] * inv;
      } else {
        uint32_t* o = reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(P.out) + grow * D + rd0);
#pragma unroll
        for (int i = 0; i < D / 16; ++i) o[i] = pack_bf16(acc[2 * i] * inv, acc[2 * i + 1] * inv);
      }
      if (P.lse && (tid & 7) == 0) P.lse[grow] = (Mq + log2f(Ls)) * static_cast<float>(kLn2);
    } else {
      float* o = P.ws_o + (grow * P.max_chunks + chunk) * D + rd0;
#pragma unroll
      for (int i = 0; i < D / 8; ++i) o[i] = acc[i];
      if ((tid & 7) == 0) P.ws_ml[grow * P.max_chunks + chunk] = make_float2(Mq, Ls);
    }
  }
}

// Grid-mapped launch: blockIdx = (chunk + max_chunks * row group, KV head, request); workgroups
// whose chunk does not exist return at once.
template <int D>
__global__ __launch_bounds__(kAttnThreads, 2) void attn_stream_kernel(AttnParams P) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int b = blockIdx.z;
  const int q0 = P.q_offsets[b];
  int n = P.q_offsets[b + 1] - q0;
  n = n > kMaxQ ? kMaxQ : n;
  stream_item<D>(P, smem, b, blockIdx.y, blockIdx.x % P.max_chunks, blockIdx.x / P.max_chunks, q0, n, P.ctx_len[b]);
}

constexpr int kPlanMaxB = 128;

// ----------------------------------------------------------------------------------
// Row-split variant for requests with more than 32 query rows per KV head (GQA groups
// times several drafts, draft trees).  The NW waves of a workgroup stage 64-token tiles
// cooperatively (double-buffered in LDS) and every wave owns one block of 32 query rows,
// for which it sees every token: no cross-wave merge is needed.
// ----------------------------------------------------------------------------------
// SL = 2 ("sliced"): the workgroup owns 32 * NW / 2 query rows and stages 128-token tiles; waves w and w + NW/2
// share a block of 32 rows, the first computing the lower 64 tokens of every staged tile, the second the upper 64,
// and they merge their results through LDS at the end.  It fills the chip from half as many (request, KV head,
// 256-row group) triples as SL = 1 without cutting the context (no partial results in memory, no combine kernel).
template <int D, int NW, int SL = 1>
struct RowsCfg {
  static constexpr int kTc = 64;                           // tokens one wave computes per step
  static constexpr int kT = kTc * SL;                      // tokens per staged tile
  static constexpr int kThreads = NW * 64;
  static constexpr int kCh = D / 8;
  static constexpr int kLoads = kT * kCh / kThreads;       // 16-byte loads per thread per tensor
  static constexpr int kTpt = kLoads;                      // consecutive tokens a thread transposes
  static constexpr int kKStride = D * 2 + 16;
  static constexpr int kKBytes = kT * kKStride;
  static constexpr int kVStride = kT * 2 + 16;
  static constexpr int kVRows = D;                         // rows in storage order, see AttnCfg
  static constexpr int kVBytes = kVRows * kVStride;
  static constexpr int kStage = kKBytes + kVBytes;
  static constexpr int kMaxChunkPages = NW == 8 ? 1024 : 512;   // a chunk spans at most 16384 (8192) tokens
  static constexpr int kPagePad = 32;                      // page-table entries kept past a chunk's last page
  // behind the two stages: ancestor masks, parents, page table
  static constexpr int meta_bytes(bool wide) { return wide ? kMaxQWide * 16 + kMaxQWide * 4 : kMaxQ * 8 + kMaxQ * 4; }
  static constexpr int lds_bytes(bool wide) { return 2 * kStage + meta_bytes(wide) + (kMaxChunkPages + kPagePad) * 4; }
  static constexpr int kLds = lds_bytes(false);
  static_assert(kTpt == 4 || kTpt == 2, "unsupported tile/thread combination");
};

// One work item of the row-split body: (request b, KV head kvh, context chunk `chunk` of `nchunks`, row group
// rg).  The request's context is cut into nchunks pieces of cb tokens (a multiple of the tile).  Every return
// below is workgroup-uniform up to the last barrier.
// WIDE: up to 128 query nodes per request (two mask words per node) instead of 64.  SL: see RowsCfg.
template <int D, int NW, bool WIDE = false, int SL = 1>
__device__ __forceinline__ void rows_item(const AttnParams& P, unsigned char* smem, int b, int kvh, int chunk, int rg,
                                          int nchunks, int cb, int q0, int n, int ctx) {
  using C = AttnCfg<D>;
  using RC = RowsCfg<D, NW, SL>;
  constexpr int kRowWaves = NW / SL;            // waves with row blocks of their own
  const int tid = static_cast<int>(threadIdx.x) + opaque_zero(), lane = tid & 63, wave = tid >> 6;
  __builtin_assume(tid >= 0 && tid < RC::kThreads);
  const int ln = lane & 31, lh = lane >> 5;

  if (n <= 0) return;
  const int L = ctx + n;
  const int R = n * P.G;
  const int row0 = rg * (32 * kRowWaves);
  if (row0 >= R) return;
  if (chunk >= nchunks) return;
  const int t_begin = chunk * cb;
  if (t_begin >= L) return;                     // rounding the chunk up to whole tiles can empty the last one
  const int t_end = min(L, t_begin + cb);
  const int ntiles = (t_end - t_begin + RC::kT - 1) / RC::kT;

  constexpr int kNodes = WIDE ? kMaxQWide : kMaxQ;
  constexpr int kWords = WIDE ? 2 : 1;
  unsigned long long* sh_anc = reinterpret_cast<unsigned long long*>(smem + 2 * RC::kStage);          // [kNodes][kWords]
  int* sh_par = reinterpret_cast<int*>(smem + 2 * RC::kStage + kNodes * kWords * 8);                  // [kNodes]
  int* sh_pages = reinterpret_cast<int*>(smem + 2 * RC::kStage + RC::meta_bytes(WIDE));               // [kMaxChunkPages]

  const bool touches_drafts = t_end > ctx;
  if (touches_drafts) {
    if (P.parent) {
      if (tid < kNodes) sh_par[tid] = (tid < n) ? P.parent[q0 + tid] : -1;
      __syncthreads();
    }
    if (tid < kNodes) {
      unsigned long long mask = 0, mask_hi = 0;
      if (tid < n) {
        if (P.parent) {
          int a = tid;
          for (int g = 0; g <= tid && a >= 0; ++g) {
            if (WIDE && a >= 64) mask_hi |= 1ull << (a - 64);
            else mask |= 1ull << a;
            const int p = sh_par[a];
            a = (p >= a || p < -1) ? -1 : p;
          }
        } else if (WIDE && tid >= 64) {
          mask = ~0ull;
          mask_hi = (2ull << (tid - 64)) - 1ull;
        } else {
          mask = (2ull << tid) - 1ull;
        }
      }
      sh_anc[tid * kWords] = mask;
      if (WIDE) sh_anc[tid * kWords + 1] = mask_hi;
    }
    __syncthreads();
  }

  // ---- this wave's 32 query rows ----
  const int slice = SL == 1 ? 0 : wave / kRowWaves;          // which 64 tokens of a staged tile this wave computes
  const int wrow0 = row0 + 32 * (wave % kRowWaves);
  const bool active = wrow0 < R;                // wave-uniform
  const int row = wrow0 + ln;
  const bool valid = row < R;
  const int node = valid ? row / P.G : 0;
  const int gq = valid ? row % P.G : 0;
  const unsigned long long my_anc = (touches_drafts && valid) ? sh_anc[node * kWords] : 0ull;
  const unsigned long long my_anc_hi = (WIDE && touches_drafts && valid) ? sh_anc[node * kWords + 1] : 0ull;
  const int64_t grow = static_cast<int64_t>(q0 + node) * P.Hq + kvh * P.G + gq;
  bf16x8 qf[C::kQKSteps];
  {
    const uint16_t* qp = P.q + grow * D + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < C::kQKSteps; ++ks) {
      u32x4 v = zero4();
      if (valid) v = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
      qf[ks] = as_bf16x8(v);
    }
  }
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 oacc[C::kDBlocks];
#pragma unroll
  for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;

  // ---- cooperative tile loads ----
  const int32_t* bt = P.block_table + static_cast<int64_t>(b) * P.max_pages;
  const int64_t page_elems = static_cast<int64_t>(P.Hkv) * kPage * D;
  const int64_t head_off = static_cast<int64_t>(kvh) * kPage * D;
  const int vc = tid % RC::kCh;                 // V: 16-byte chunk of the token row
  const int vg = tid / RC::kCh;                 // V: group of kTpt consecutive tokens
  const int vtok0 = vg * RC::kTpt;              // first of them within the tile
  // two register sets: while tile t is computed from LDS, tile t+1 waits in one set and tile
  // t+2 is in flight into the other, i.e. two tiles of global loads are outstanding per workgroup
  u32x4 krA[RC::kLoads], vrA[RC::kLoads], krB[RC::kLoads], vrB[RC::kLoads];

  // Page ids of the whole chunk go to LDS once, so that the tile loads depend on no global read.
  const int lp0 = t_begin / kPage;
  const int np = (t_end + kPage - 1) / kPage - lp0;          // >= 1 pages touched by this chunk
  // (entries past the chunk's last page repeat it: tile numbers past the end need no clamp)
  for (int i = tid; i < np + RC::kPagePad; i += RC::kThreads) sh_pages[i] = bt[lp0 + min(i, np - 1)];
  __syncthreads();

  // Loads are unconditional (addresses clamped to the chunk's last page): positions past the
  // end are masked out of the scores, and their V values are zeroed when staged.
  // Every load instruction of a wave touches one cache page, so the page id is wave-uniform
  // (scalar base) and only a small per-lane offset lives in a vector register.
  constexpr int kTokPerLoadWg = RC::kThreads / RC::kCh;               // tokens one load j of the workgroup covers
  const int k_tok_in_load = tid / RC::kCh;                            // token of this lane within load j
  const int k_lane_off = (k_tok_in_load % kPage) * D + (tid % RC::kCh) * 8;
  const int k_page_in_load = k_tok_in_load / kPage;                   // wave-uniform
  const int v_lane_off = (vtok0 % kPage) * D + vc * 8;
  // The page ids of tile t are read from LDS right after the loads of tile t-1 were issued, a whole tile step
  // before they are needed: the address of a load then waits on no LDS round trip.
  int pg[RC::kLoads + 1];
  auto fetch_pages = [&](int t) {
    const int* tp = sh_pages + min(RC::kT * t / kPage, np + RC::kPagePad - RC::kT / kPage);
#pragma unroll
    for (int j = 0; j < RC::kLoads; ++j) pg[j] = tp[(j * kTokPerLoadWg) / kPage + k_page_in_load];
    pg[RC::kLoads] = tp[vtok0 / kPage];
  };
  auto issue_loads = [&](u32x4 (&kr)[RC::kLoads], u32x4 (&vr)[RC::kLoads]) {
#pragma unroll
    for (int j = 0; j < RC::kLoads; ++j) {
      const int page = __builtin_amdgcn_readfirstlane(pg[j]);
      const uint16_t* base = P.k_pool + page * page_elems + head_off;
      kr[j] = *reinterpret_cast<const u32x4*>(base + k_lane_off);
    }
    const int page = __builtin_amdgcn_readfirstlane(pg[RC::kLoads]);
    const uint16_t* vp = P.v_pool + page * page_elems + head_off + v_lane_off;
#pragma unroll
    for (int i = 0; i < RC::kTpt; ++i) vr[i] = *reinterpret_cast<const u32x4*>(vp + i * D);
  };
  // issue the loads of tile t (tiles are issued in order: t is the one whose page ids were fetched last)
  auto issue_tile = [&](int t, u32x4 (&kr)[RC::kLoads], u32x4 (&vr)[RC::kLoads]) __attribute__((always_inline)) {
    issue_loads(kr, vr);
    fetch_pages(t + 1);
  };

  auto store_tile = [&](int stage, int t, u32x4 (&kr)[RC::kLoads], u32x4 (&vr)[RC::kLoads]) {
    unsigned char* k_lds = smem + stage * RC::kStage;
    unsigned char* v_lds = k_lds + RC::kKBytes;
#pragma unroll
    for (int j = 0; j < RC::kLoads; ++j) {
      const int tk = j * (RC::kThreads / RC::kCh) + tid / RC::kCh;
      *reinterpret_cast<u32x4*>(k_lds + tk * RC::kKStride + (tid % RC::kCh) * 16) = kr[j];
    }
    // transposed V: token order inside each 16-token group follows the MFMA operand layout
    const int s16 = vtok0 / 16, u = vtok0 % 16;
    const int a4 = u >> 2, sub = u & 3;
    const int pos = 8 * (a4 & 1) + 4 * (a4 >> 1) + sub;
    const int col = (16 * s16 + pos) * 2;
    // never multiply stale cache slots (past ctx+n) into O: stage them as zeros
    if (t_begin + RC::kT * (t + 1) > L) {                     // only the last tile (and the ones past it)
      const int left = L - (t_begin + RC::kT * t + vtok0);    // tokens of this thread that exist
#pragma unroll
      for (int i = 0; i < RC::kTpt; ++i)
        if (i >= left) vr[i] = zero4();
    }
    // V goes to LDS as fp16 (the weights P are fp16 too: 11 significant bits in ONE matrix term)
#pragma unroll
    for (int i = 0; i < RC::kTpt; ++i)
#pragma unroll
      for (int k = 0; k < 4; ++k) vr[i][k] = bf16x2_to_f16x2(vr[i][k]);
    const u32x4 w0 = vr[0], w1 = vr[1];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const uint32_t sel = half ? 0x07060302u : 0x05040100u;
        const int vrow = (2 * k + half) * (D / 8) + vc;
        unsigned char* dst = v_lds + vrow * RC::kVStride + col;
        if constexpr (RC::kTpt == 4) {
          const uint32_t w2k = vr[2][k], w3k = vr[3][k];
          uint2 o;
          o.x = __builtin_amdgcn_perm(w1[k], w0[k], sel);
          o.y = __builtin_amdgcn_perm(w3k, w2k, sel);
          *reinterpret_cast<uint2*>(dst) = o;
        } else {
          *reinterpret_cast<uint32_t*>(dst) = __builtin_amdgcn_perm(w1[k], w0[k], sel);
        }
      }
    }
  };

  // One 64-token tile = one online-softmax step in two parts (scores, output) that share these registers.
  f32x16 sacc[2];
  f16x8 ph, va[C::kDBlocks];
  float m_safe = 0.f, m_next = -INFINITY, alpha = 1.f, psum = 0.f;
  auto v_frag = [&](int stage, int chunk, int db) {      // chunk = 16-token group 0..3 of the tile
    const unsigned char* v_rd = smem + stage * RC::kStage + RC::kKBytes + ln * RC::kVStride + 16 * lh + 2 * RC::kTc * slice;
    return __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(v_rd + 32 * db * RC::kVStride + 32 * chunk));
  };
  // P^T as fp16 (weights lie in [0, 2^8]: 11 significant bits, against 8 of bf16, keep the output's error at the
  // level of its own bf16 rounding with a single matrix term), 16 tokens at a time
  auto p_chunk = [&](int chunk, f16x8& dst) __attribute__((always_inline)) {
    const int tb = chunk >> 1, sg = chunk & 1;
    u32x4 hw;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float p0 = fast_exp2(fmaf(sacc[tb][8 * sg + 2 * j], P.c, -m_safe));
      const float p1 = fast_exp2(fmaf(sacc[tb][8 * sg + 2 * j + 1], P.c, -m_safe));
      psum += p0 + p1;
      hw[j] = pack_f16(p0, p1);
    }
    dst = __builtin_bit_cast(f16x8, hw);
  };

  // First half: S = K Q^T (operand reads from LDS run two steps ahead of the matrix instructions that consume
  // them), mask, row maxima, rescale, the weights of the first 16 tokens.
  auto tile_scores = [&](int stage, int t) __attribute__((always_inline)) {
    const unsigned char* k_lds = smem + stage * RC::kStage + slice * RC::kTc * RC::kKStride;
    const int tok0 = t_begin + RC::kT * t + RC::kTc * slice;
    const unsigned char* k_rd = k_lds + ln * RC::kKStride + 16 * lh;
    auto k_frag = [&](int ks, int tb) {
      return as_bf16x8(*reinterpret_cast<const u32x4*>(k_rd + 32 * tb * RC::kKStride + 32 * ks));
    };
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[tb][r] = 0.f;
    // three operand slots in rotation: the slot refilled at step ks was last read by the MFMAs
    // of step ks-1, never by the ones just issued
    bf16x8 ka[3][2];
    ka[0][0] = k_frag(0, 0); ka[0][1] = k_frag(0, 1);
    ka[1][0] = k_frag(1, 0); ka[1][1] = k_frag(1, 1);
#pragma unroll
    for (int ks = 0; ks < C::kQKSteps; ++ks) {
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 2 < C::kQKSteps) {
        ka[(ks + 2) % 3][0] = k_frag(ks + 2, 0);
        ka[(ks + 2) % 3][1] = k_frag(ks + 2, 1);
      }
      sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks % 3][0], qf[ks], sacc[0], 0, 0, 0);
      sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks % 3][1], qf[ks], sacc[1], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // V^T operand of the first 16 tokens is fetched while the scores are reduced
#pragma unroll
    for (int db = 0; db < C::kDBlocks; ++db) va[db] = v_frag(stage, 0, db);

    if (tok0 + RC::kTc > ctx) {                  // tile reaches the drafts or the end: apply the mask
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int pos = tok0 + 32 * tb + 8 * (r >> 2) + 4 * lh + (r & 3);
          // branch-free on purpose: bitwise ops, no short-circuit control flow around the accumulator
          const unsigned long long word = (WIDE && ((pos - ctx) & 64)) ? my_anc_hi : my_anc;
          const bool ok = (pos < ctx) | ((pos < L) & (((word >> ((pos - ctx) & 63)) & 1ull) != 0ull));
          sacc[tb][r] = ok ? sacc[tb][r] : -INFINITY;
        }
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sacc[tb][r]);
    tmax *= P.c;                                   // c > 0: the maximum commutes with the scaling
    tmax = half_max(tmax);
    // The running maximum only has to bound the exponents: it follows the true maximum when that is first
    // finite or has grown by more than 8 (weights then reach 2^8 at most, exact in fp16 and fp32); the
    // accumulator is rescaled on those steps alone, and the final O / l is the same quotient either way.
    m_next = fmaxf(m_run, tmax);
    if (m_run != -INFINITY && tmax <= m_run + 8.f) m_next = m_run;
    m_safe = (m_next == -INFINITY) ? 0.f : m_next;
    alpha = fast_exp2(m_run - m_safe);
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    psum = 0.f;
    p_chunk(0, ph);
  };

  // Second half: O += P V, 16 tokens at a time, with the exponentials of the next 16 tokens between the
  // matrix instructions of the current ones.
  auto tile_output = [&](int stage) __attribute__((always_inline)) {
#pragma unroll
    for (int chunk = 0; chunk < 4; ++chunk) {
      __builtin_amdgcn_sched_barrier(0);
      f16x8 vn[C::kDBlocks];
      f16x8 nh;
      if (chunk + 1 < 4) {
#pragma unroll
        for (int db = 0; db < C::kDBlocks; ++db) vn[db] = v_frag(stage, chunk + 1, db);
      }
#pragma unroll
      for (int db = 0; db < C::kDBlocks; ++db)
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[db], ph, oacc[db], 0, 0, 0);
      if (chunk + 1 < 4) {
        p_chunk(chunk + 1, nh);
        // A wave issues in order: matrix instructions queued back to back would hold the weights of the next
        // 16 tokens behind them.  One matrix instruction, one operand read, then a quarter of the vector work.
#pragma unroll
        for (int i = 0; i < C::kDBlocks; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
        }
        ph = nh;
#pragma unroll
        for (int db = 0; db < C::kDBlocks; ++db) va[db] = vn[db];
      }
    }
    l_run = l_run * alpha + psum;
    m_run = m_next;
  };

  // ---- pipeline: tile t is computed from LDS while tile t+1 sits in registers ----
  // Loads and LDS stores are issued unconditionally, also for tile numbers past the end (their addresses are
  // clamped to the chunk's last page, their V rows staged as zeros, and they are never computed): with the
  // same number of loads outstanding on every path, the wait before a store covers only the older register
  // set and leaves the newer one in flight.  A branch around an issue would make that wait a full drain.
  // (a wave of the sliced variant skips a staged tile whose half for it lies past the end)
  auto mine = [&](int t) { return active && t < ntiles && t_begin + RC::kT * t + RC::kTc * slice < t_end; };
  fetch_pages(0);
  if constexpr (NW == 8 && SL == 1) {
    issue_tile(0, krA, vrA);
    issue_tile(1, krB, vrB);
    store_tile(0, 0, krA, vrA);
    issue_tile(2, krA, vrA);
    __syncthreads();
    for (int t = 0; t < ntiles; t += 2) {
      // LDS stage 0 holds tile t, set B tile t+1, set A tile t+2
      if (mine(t)) { tile_scores(0, t); tile_output(0); }
      store_tile(1, t + 1, krB, vrB);
      issue_tile(t + 3, krB, vrB);
      __syncthreads();
      // LDS stage 1 holds tile t+1, set A tile t+2, set B tile t+3
      if (mine(t + 1)) { tile_scores(1, t + 1); tile_output(1); }
      store_tile(0, t + 2, krA, vrA);
      issue_tile(t + 4, krA, vrA);
      __syncthreads();
    }
  } else {
    // Four waves, two workgroups per compute unit: one register set (one tile of loads in flight per
    // workgroup; the other workgroup covers the rest of the latency), which leaves the registers for it.
    issue_tile(0, krA, vrA);
    store_tile(0, 0, krA, vrA);
    issue_tile(1, krA, vrA);
    __syncthreads();
    for (int t = 0; t < ntiles; t += 2) {
      if (mine(t)) { tile_scores(0, t); tile_output(0); }
      store_tile(1, t + 1, krA, vrA);
      issue_tile(t + 2, krA, vrA);
      __syncthreads();
      if (mine(t + 1)) { tile_scores(1, t + 1); tile_output(1); }
      store_tile(0, t + 2, krA, vrA);
      issue_tile(t + 3, krA, vrA);
      __syncthreads();
    }
  }

  l_run = half_sum(l_run);
  if constexpr (SL == 2) {
    // ---- the wave that took the upper halves of the tiles hands (m, l, O) to the one that took the lower halves
    // (the tile memory is free: the loop ended with a barrier); accumulator registers go over as they are, one
    // 256-byte row of LDS per register ----
    float* xo = reinterpret_cast<float*>(smem) + (wave % kRowWaves) * (C::kDBlocks * 16 + 2) * 64;
    if (slice == 1 && active) {
#pragma unroll
      for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) xo[(db * 16 + r) * 64 + lane] = oacc[db][r];
      xo[(C::kDBlocks * 16) * 64 + lane] = m_run;
      xo[(C::kDBlocks * 16 + 1) * 64 + lane] = l_run;
    }
    __syncthreads();
    if (slice == 1) return;
    if (active) {
      const float m2 = xo[(C::kDBlocks * 16) * 64 + lane], l2 = xo[(C::kDBlocks * 16 + 1) * 64 + lane];
      const float M = fmaxf(m_run, m2);
      const float f1 = m_run == -INFINITY ? 0.f : fast_exp2(m_run - M);
      const float f2 = m2 == -INFINITY ? 0.f : fast_exp2(m2 - M);
#pragma unroll
      for (int db = 0; db < C::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = oacc[db][r] * f1 + xo[(db * 16 + r) * 64 + lane] * f2;
      l_run = l_run * f1 + l2 * f2;
      m_run = M;
    }
  }
  // ---- write this wave's rows ----
  if (!active) return;
  if (!valid) return;
  // The weights were truncated to fp16 (round toward zero): every one is low by a factor that is uniform in
  // [0, 2^-11], 2^-12 on average, while the denominator l was summed from the unrounded weights.  The
  // average is put back here; what remains is the zero-mean part (2^-12 at most per weight).
  constexpr float kRtzFix = 1.f + 1.f / 4096.f;
  // eight consecutive head dimensions at a time (acc_dim0)
  constexpr int kA = D / 64, kQ = 256 / D;
  const float oscale = nchunks == 1 ? kRtzFix / l_run : kRtzFix;
  float* part = P.ws_o + (grow * P.max_chunks + chunk) * D;
#pragma unroll
  for (int am = 0; am < kA; ++am)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = oacc[j / kQ][4 * ((j % kQ) * kA + am) + c] * oscale;
      const int d = acc_dim0<D>(am, c, lh);
      if (nchunks != 1 || P.out_f32) {
        // fp32 rows: the two half-waves exchange halves of their eight values, so that one store instruction
        // writes 32 contiguous bytes per row (lane ln: 16 bytes, lane ln + 32: the next 16) instead of 16
        float lo4[4], hi4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x[i]), __float_as_uint(x[4 + i]), false, false);
          lo4[i] = __uint_as_float(r[0]);          // dims d0 .. of the lower half-wave's group: first / second four
          hi4[i] = __uint_as_float(r[1]);          // dims d0 .. of the upper half-wave's group
        }
        float* o = (nchunks != 1 ? part : static_cast<float*>(P.out) + grow * D) + acc_dim0<D>(am, c, 0) + 4 * lh;
        *reinterpret_cast<float4*>(o) = make_float4(lo4[0], lo4[1], lo4[2], lo4[3]);
        *reinterpret_cast<float4*>(o + 32) = make_float4(hi4[0], hi4[1], hi4[2], hi4[3]);
      } else {
        u32x4 o;
        o[0] = pack_bf16(x[0], x[1]); o[1] = pack_bf16(x[2], x[3]);
        o[2] = pack_bf16(x[4], x[5]); o[3] = pack_bf16(x[6], x[7]);
        *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(P.out) + grow * D + d) = o;
      }
    }
  if (nchunks == 1) {
    if (P.lse && lh == 0) P.lse[grow] = (m_run + log2f(l_run)) * static_cast<float>(kLn2);
  } else if (lh == 0) {
    P.ws_ml[grow * P.max_chunks + chunk] = make_float2(m_run, l_run);
  }
}

template <int D, int NW, bool WIDE, int SL>
__global__ __launch_bounds__(NW * 64, (NW == 4 ? 2 : 1)) void attn_rows_kernel(AttnParams P) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  if (P.xcd_swizzle) {
    // Workgroups go to the 8 XCDs in turn.  With several row groups per (request, KV head) pair, renumber so that
    // the row groups of a pair run on one XCD at the same time: the second read of the pair's K/V hits in that L2.
    const unsigned total = gridDim.x * gridDim.y * gridDim.z;           // a multiple of 8 (checked by the host)
    const unsigned linear = bx + gridDim.x * (by + gridDim.y * bz);
    const unsigned logical = (linear % 8u) * (total / 8u) + linear / 8u;
    bx = logical % gridDim.x;
    by = (logical / gridDim.x) % gridDim.y;
    bz = logical / (gridDim.x * gridDim.y);
  }
  const int b = static_cast<int>(bz);
  const int chunk = static_cast<int>(bx) % P.max_chunks, rg = static_cast<int>(bx) / P.max_chunks;
  const int q0 = P.q_offsets[b];
  int n = P.q_offsets[b + 1] - q0;
  n = n > (WIDE ? kMaxQWide : kMaxQ) ? (WIDE ? kMaxQWide : kMaxQ) : n;
  const int ctx = P.ctx_len[b];
  const int L = ctx + n;
  const int nchunks = max(1, (L + P.chunk_tokens - 1) / P.chunk_tokens);
  const int cb = (((L + nchunks - 1) / nchunks) + RowsCfg<D, NW, SL>::kT - 1) & ~(RowsCfg<D, NW, SL>::kT - 1);
  rows_item<D, NW, WIDE, SL>(P, smem, b, static_cast<int>(by), chunk, rg, nchunks, cb, q0, n, ctx);
}

// Sorted-work-list launch for batches of up to kPlanMaxB requests with ragged lengths.  The grid
// is two workgroups per compute unit; every workgroup derives the same list of work items
// (request, chunk, KV head) from the lengths on the device, ordered by decreasing number of tiles
// a wave streams per item, and takes one item per round of gridDim.x items (in workgroup order on even
// rounds, reversed on odd ones): long items start first, short ones fill the tail, and no workgroup is
// launched for chunks that do not exist.
// An item runs the token-split body or, for requests with many query rows, the row-split body.
template <int D>
__global__ __launch_bounds__(kAttnThreads, 2) void attn_stream_list_kernel(AttnParams P) {
  using RC = RowsCfg<D, 4>;
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int sh_first[kPlanMaxB + 1];        // first item of the request at sorted position s
  // the request at sorted position s: first query row (below 2^16) | nodes << 16 | request << 24, and its context
  // length: an item starts without a round trip to global memory for them
  __shared__ int sh_meta[kPlanMaxB], sh_ctx[kPlanMaxB];
  static_assert(kPlanMaxB <= 128 && kMaxQ <= 64, "request and node count share one word with the first query row");
  const int tid = threadIdx.x;
  int* key = reinterpret_cast<int*>(smem);       // scratch in the tile memory, dead before the first item
  int* cnt = key + kPlanMaxB;
  int my_key = -1, my_cnt = 0, my_meta = 0, my_ctx = 0;
  if (tid < P.B) {
    const int q0 = P.q_offsets[tid];
    int n = P.q_offsets[tid + 1] - q0;
    n = n > kMaxQ ? kMaxQ : (n < 0 ? 0 : n);
    const int ctx = P.ctx_len[tid];
    my_meta = q0 | (n << 16) | (tid << 24);
    my_ctx = ctx;
    if (n > 0) {
      const int L = ctx + n;
      const int nch = request_chunks(P, L, n);
      my_key = (request_units(P, L, n) + nch - 1) / nch;   // length of one item of this request
      my_cnt = nch * P.Hkv;
    }
  }
  if (tid < kPlanMaxB) { key[tid] = my_key; cnt[tid] = my_cnt; }
  __syncthreads();
  if (tid < P.B) {
    int rank = 0, first = 0;
    for (int j = 0; j < P.B; ++j) {
      const int kj = key[j];
      const bool before = kj > my_key || (kj == my_key && j < tid);
      rank += before ? 1 : 0;
      first += before ? cnt[j] : 0;
    }
    sh_meta[rank] = my_meta;
    sh_ctx[rank] = my_ctx;
    sh_first[rank] = first;
    if (rank == P.B - 1) sh_first[P.B] = first + my_cnt;
  }
  __syncthreads();
  const int total = sh_first[P.B];
  // Round r hands out items r*G .. r*G+G-1 (G workgroups), in workgroup order on even rounds and in reverse
  // on odd ones: the workgroup that got the longest item of one round gets the shortest of the next.
  for (int round = 0;; ++round) {
    const int slot = (round & 1) ? static_cast<int>(gridDim.x - 1 - blockIdx.x) : static_cast<int>(blockIdx.x);
    const int item = round * static_cast<int>(gridDim.x) + slot;
    if (item >= total) break;
    int lo = 0, hi = P.B;                         // largest s with sh_first[s] <= item
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (sh_first[mid] <= item) lo = mid; else hi = mid;
    }
    const int meta = sh_meta[lo];
    const int b = meta >> 24, q0 = meta & 0xffff, n = (meta >> 16) & 0xff, ctx = sh_ctx[lo];
    const int local = item - sh_first[lo];
    const int L = ctx + n;
    const int nch = request_chunks(P, L, n);
    const int cb = (((L + nch - 1) / nch) + RC::kT - 1) & ~(RC::kT - 1);
    // (a chunk longer than the row-split body's page table in LDS stays with the token-split body)
    if (list_uses_rows(P, n) && cb <= RC::kMaxChunkPages * kPage) rows_item<D, 4>(P, smem, b, local % P.Hkv, local / P.Hkv, 0, nch, cb, q0, n, ctx);
    else stream_item<D>(P, smem, b, local % P.Hkv, local / P.Hkv, 0, q0, n, ctx);
    __syncthreads();                              // the tile memory is reused by the next item
  }
}

// Merge the per-chunk partials of every (query row, head) that spans several chunks.
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnParams P) {
  constexpr int kPer = D / 32;
  // blockIdx.y = request; 8 (query node, head) rows of it per workgroup, 32 threads per row
  const int b = blockIdx.y;
  const int q0 = P.q_offsets[b];
  int n = P.q_offsets[b + 1] - q0;
  n = n > P.n_cap ? P.n_cap : n;
  const int local = blockIdx.x * 8 + (threadIdx.x >> 5);
  if (local >= n * P.Hq) return;
  const int64_t grow = static_cast<int64_t>(q0) * P.Hq + local;
  const int d0 = (threadIdx.x & 31) * kPer;
  const int L = P.ctx_len[b] + n;
  const int nchunks = request_chunks(P, L, n);
  if (nchunks == 1) return;
  float M = -INFINITY;
  for (int c = 0; c < nchunks; ++c) M = fmaxf(M, P.ws_ml[grow * P.max_chunks + c].x);
  float acc[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) acc[i] = 0.f;
  float W = 0.f;
  for (int c = 0; c < nchunks; ++c) {
    const float2 ml = P.ws_ml[grow * P.max_chunks + c];
    if (ml.x == -INFINITY) continue;
    const float f = fast_exp2(ml.x - M);
    W += ml.y * f;
    const float* o = P.ws_o + (grow * P.max_chunks + c) * D + d0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) acc[i] += o[i] * f;
  }
  const float inv = 1.f / W;
  if (P.out_f32) {
    float* o = static_cast<float*>(P.out) + grow * D + d0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) o[i] = acc[i] * inv;
  } else {
    uint16_t* o = static_cast<uint16_t*>(P.out) + grow * D + d0;
#pragma unroll
    for (int i = 0; i < kPer; i += 2) *reinterpret_cast<uint32_t*>(o + i) = pack_bf16(acc[i] * inv, acc[i + 1] * inv);
  }
  if (P.lse && (threadIdx.x & 31) == 0) P.lse[grow] = (M + log2f(W)) * static_cast<float>(kLn2);
}

// ----------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------
constexpr int kListMaxChunks = 16;

// Development knobs for sweeps, compiled in only with -DSPECV_DEV_KNOBS (normal builds read no
// environment variable and keep no state between calls).
#ifdef SPECV_DEV_KNOBS
static long dev_knob(const char* name, long fallback) {
  const char* e = getenv(name);
  return e ? atol(e) : fallback;
}
#else
static long dev_knob(const char*, long fallback) { return fallback; }
#endif

AttnPlan make_attn_plan(const AttnArgs& a) {
  AttnPlan p;
  p.tau = 0;
  p.wide = a.max_q > kMaxQ ? 1 : 0;
  const int G = a.Hq / a.Hkv;
  const int max_rows = a.max_q * G;
  const int64_t max_tok0 = static_cast<int64_t>(a.max_pages) * a.page;
  const bool ragged0 = a.kv_hint > 0 && a.kv_hint * 100 < static_cast<int64_t>(85) * a.B * max_tok0;
  // Up to 64 query rows per KV head the token-split body streams as fast as memory delivers; beyond, its
  // waves (one per 32-row block, each staging every tile for itself) are bound by their own staging and the
  // row-split body, whose waves share each staged tile, is ahead on batches of like lengths (96 rows per KV
  // head: 4.2 against 2.6 TB/s).  Ragged batches keep the token-split body and its sorted work list.
  if (max_rows <= 64 || (max_rows <= 128 && ragged0 && a.B <= kPlanMaxB)) { p.kind = 0; p.rows_per_wg = 128; }
  else if (max_rows <= 128 || a.D != 128) { p.kind = 1; p.rows_per_wg = 128; }
  else { p.kind = 2; p.rows_per_wg = 256; }
  // Few (request, KV head) pairs with many rows each: 256-row workgroups would have to cut the context to fill
  // the chip (partial results through memory and a combine kernel).  The sliced variant gives every pair twice
  // the workgroups instead - 128 rows each, the token halves of every tile split between two waves - when one
  // such workgroup per compute unit covers the batch.
  if (p.kind == 2) {
    const int64_t groups256 = static_cast<int64_t>(a.B) * a.Hkv * ((max_rows + 255) / 256);
    const int64_t groups128 = static_cast<int64_t>(a.B) * a.Hkv * ((max_rows + 127) / 128);
    const int n_cu = current_device_cus();
    if (groups256 * 4 <= 3 * static_cast<int64_t>(n_cu) && groups128 <= n_cu + n_cu / 4) { p.kind = 3; p.rows_per_wg = 128; }
  }
  const long force_kind = dev_knob("SPECV_ATTN_KIND", -1);            // force a kernel family
  if (force_kind == 1) { p.kind = 1; p.rows_per_wg = 128; }
  if (force_kind == 2 && a.D == 128) { p.kind = 2; p.rows_per_wg = 256; }
  if (force_kind == 0) { p.kind = 0; p.rows_per_wg = 128; }
  if (force_kind == 3 && a.D == 128 && max_rows > 128) { p.kind = 3; p.rows_per_wg = 128; }
  // more than 64 query nodes per request (two mask words per node): the row-split kernels only
  if (p.wide && p.kind == 0) { p.kind = 1; p.rows_per_wg = 128; }
  p.row_groups = (max_rows + p.rows_per_wg - 1) / p.rows_per_wg;
  const bool token_split = (p.kind == 0);
  const int gran = token_split ? kTile : (p.kind == 3 ? 128 : 64);              // chunks are whole tiles
  const int64_t max_tok = static_cast<int64_t>(a.max_pages) * a.page;
  int64_t tok = a.kv_hint > 0 ? a.kv_hint : static_cast<int64_t>(a.B) * max_tok;
  // Chunk length.  Every workgroup pays a fixed prologue/epilogue (and, when a request is split, a
  // partial-result round trip proportional to its query rows), so chunks are as long as two
  // limits allow: (a) about one workgroup per compute unit should exist, (b) one wave should not
  // stream more than ~40 tiles in sequence, or the longest workgroup sets the kernel's duration.
  const long jobs_knob = dev_knob("SPECV_ATTN_JOBS", 0);
  const int64_t jobs_target = jobs_knob > 0 ? jobs_knob : (p.kind == 1 ? 512 : 256);   // 4-wave bodies: two per compute unit
  int64_t chunk = (tok * a.Hkv * p.row_groups + jobs_target - 1) / jobs_target;
  if (token_split && jobs_knob <= 0) {
    // waves that share one query block (pair) and therefore split its tiles
    const int nslice = max_rows <= 32 ? 4 : (max_rows <= 64 ? 2 : 1);
    const int64_t cap = static_cast<int64_t>(40) * kTile * nslice;
    if (chunk > cap) chunk = cap;
  }
  if (chunk < 256) chunk = 256;
  chunk = (chunk + gran - 1) / gran * gran;
  if (chunk > max_tok) chunk = (max_tok + gran - 1) / gran * gran;
  // the row-split kernel keeps a chunk's page ids in LDS
  const int64_t rows_chunk_cap = (p.kind >= 2) ? 16384 : 8192;
  if (!token_split && chunk > rows_chunk_cap) chunk = rows_chunk_cap;
  if (chunk < gran) chunk = gran;
  p.chunk_tokens = static_cast<int>(chunk);
  p.max_chunks = static_cast<int>((max_tok + chunk - 1) / chunk);
  if (p.max_chunks < 1) p.max_chunks = 1;
  // Small batches whose lengths are ragged run the token-split kernel from a sorted work list built
  // on the device (the lengths are device data); there chunks are cut by tiles per wave, not by
  // tokens.  The list costs every workgroup one extra round of dependent loads (~5 us per launch),
  // which only pays when lengths differ: the caller's total-token hint against batch x longest
  // request says whether they do.
  const bool ragged = a.kv_hint > 0 && a.kv_hint * 100 < static_cast<int64_t>(85) * a.B * max_tok;
  // (the list kernel packs a request's first query row into 16 bits)
  int tau = (token_split && a.B <= kPlanMaxB && a.total_q < 65536 && ragged) ? 44 : 0;   // with the alternating hand-out below: 40-48 measured best
  const long tau_knob = dev_knob("SPECV_ATTN_TAU", -1);   // 0: grid-mapped launch
  if (token_split && a.B <= kPlanMaxB && a.total_q < 65536 && tau_knob >= 0 && tau_knob <= 255) tau = static_cast<int>(tau_knob);
  if (jobs_knob > 0) tau = 0;
  if (tau > 0) {
    // most tiles one wave can have to stream: the longest request, shared by as many waves as the
    // largest declared row count leaves per query block (requests with fewer rows get more waves)
    const int min_slice = max_rows <= 32 ? 4 : (max_rows <= 64 ? 2 : 1);
    const int64_t max_tiles = ((max_tok + kTile - 1) / kTile + min_slice - 1) / min_slice;
    const int64_t mc = (max_tiles + tau - 1) / tau;
    p.tau = tau;
    p.max_chunks = static_cast<int>(mc < 1 ? 1 : (mc > kListMaxChunks ? kListMaxChunks : mc));
  }
  return p;
}

size_t attn_workspace_bytes(const AttnArgs& a, const AttnPlan& p) {
  if (p.max_chunks <= 1) return 256;
  const size_t rows = static_cast<size_t>(a.total_q) * a.Hq;
  return rows * p.max_chunks * (a.D + 2) * sizeof(float) + 256;
}

const char* attn_plan_name(const AttnPlan& p) {
  if (p.kind == 0) return p.tau > 0 ? "attn_stream_list_kernel (device-built work list sorted by length; token-split body, row-split body from 65 query rows per KV head)"
                                    : "attn_stream_kernel (token-split body, one workgroup per request x KV head x context chunk)";
  if (p.kind == 1) return "attn_rows_kernel<4 waves> (row-split body)";
  if (p.kind == 3) return "attn_rows_kernel<8 waves, sliced> (row-split body, 128 query rows per workgroup, two waves per 32-row block)";
  return "attn_rows_kernel<8 waves> (row-split body, 256 query rows per workgroup)";
}

template <int D>
static int launch_stream(const AttnParams& P, const AttnPlan& plan, int B, int Hkv, hipStream_t stream) {
  using C = AttnCfg<D>;
  constexpr size_t kMerge = kAttnWaves * 32 * C::kORedStride * sizeof(float) + 2 * kAttnWaves * 32 * sizeof(float);
  constexpr size_t kTiles = static_cast<size_t>(kAttnWaves) * C::kWaveLds;
  static_assert(kMerge <= kTiles, "merge buffers must fit in the tile memory");
  static std::atomic<uint64_t> attr_done{0};
  if (set_lds_once(&attn_stream_kernel<D>, kTiles, attr_done) != 0) return -6;
  if (plan.tau > 0) {
    // both bodies run in this kernel: the tile memory of the larger one
    constexpr size_t kListLds = kTiles > static_cast<size_t>(RowsCfg<D, 4>::kLds) ? kTiles : static_cast<size_t>(RowsCfg<D, 4>::kLds);
    // two workgroups per compute unit: dynamic plus the kernel's static LDS (below 1664 bytes) within half of 160 KB
    static_assert(kListLds + 1664 <= 80 * 1024, "the work-list kernel must fit twice into a compute unit's LDS");
    static std::atomic<uint64_t> list_attr_done{0};
    if (set_lds_once(&attn_stream_list_kernel<D>, kListLds, list_attr_done) != 0) return -6;
    const int n_cu = current_device_cus();
    hipLaunchKernelGGL((attn_stream_list_kernel<D>), dim3(2 * n_cu), dim3(kAttnThreads), kListLds, stream, P);
    return hipGetLastError() == hipSuccess ? 0 : -6;
  }
  dim3 grid(plan.max_chunks * plan.row_groups, Hkv, B);
  hipLaunchKernelGGL((attn_stream_kernel<D>), grid, dim3(kAttnThreads), kTiles, stream, P);
  return hipGetLastError() == hipSuccess ? 0 : -6;
}

template <int D, int NW, bool WIDE, int SL = 1>
static int launch_rows_as(const AttnParams& P, const AttnPlan& plan, int B, int Hkv, hipStream_t stream) {
  using RC = RowsCfg<D, NW, SL>;
  constexpr size_t kLds = RC::lds_bytes(WIDE);
  static_assert(kLds * (NW == 4 ? 2 : 1) <= 160 * 1024, "row-split kernel: LDS per compute unit");
  static std::atomic<uint64_t> attr_done{0};
  if (set_lds_once(&attn_rows_kernel<D, NW, WIDE, SL>, kLds, attr_done) != 0) return -6;
  dim3 grid(plan.max_chunks * plan.row_groups, Hkv, B);
  hipLaunchKernelGGL((attn_rows_kernel<D, NW, WIDE, SL>), grid, dim3(RC::kThreads), kLds, stream, P);
  return hipGetLastError() == hipSuccess ? 0 : -6;
}

template <int D, int NW>
static int launch_rows(const AttnParams& P, const AttnPlan& plan, int B, int Hkv, hipStream_t stream) {
  return plan.wide ? launch_rows_as<D, NW, true>(P, plan, B, Hkv, stream) : launch_rows_as<D, NW, false>(P, plan, B, Hkv, stream);
}

int launch_attn(const AttnArgs& a, const AttnPlan& plan, hipStream_t stream) {
  if (a.B <= 0 || a.total_q <= 0) return 0;
  AttnParams P;
  P.q = static_cast<const uint16_t*>(a.q);
  P.k_pool = static_cast<const uint16_t*>(a.k_pool);
  P.v_pool = static_cast<const uint16_t*>(a.v_pool);
  P.block_table = a.block_table; P.ctx_len = a.ctx_len; P.q_offsets = a.q_offsets; P.parent = a.parent;
  P.out = a.out; P.lse = a.lse;
  const size_t rows = static_cast<size_t>(a.total_q) * a.Hq;
  P.ws_ml = static_cast<float2*>(a.workspace);
  P.ws_o = reinterpret_cast<float*>(static_cast<unsigned char*>(a.workspace) +
                                    ((rows * plan.max_chunks * sizeof(float2) + 255) / 256) * 256);
  P.B = a.B; P.Hq = a.Hq; P.Hkv = a.Hkv; P.G = a.Hq / a.Hkv; P.max_pages = a.max_pages;
  P.chunk_tokens = plan.chunk_tokens; P.max_chunks = plan.max_chunks; P.tau = plan.tau;
  // work list: from 65 query rows per KV head (three 32-row blocks) on, a request runs the row-split body
  P.list_rows_min = plan.tau > 0 ? static_cast<int>(dev_knob("SPECV_ATTN_LIST_ROWS", 65)) : 0;
  P.list_rows_units = static_cast<int>(dev_knob("SPECV_ATTN_ROWS_UNITS", 3));
  P.n_cap = plan.wide ? kMaxQWide : kMaxQ;
  P.xcd_swizzle = (plan.kind != 0 && plan.row_groups > 1 &&
                   (static_cast<int64_t>(plan.max_chunks) * plan.row_groups * a.Hkv * a.B) % 8 == 0) ? 1 : 0;
  P.c = a.scale * kLog2e;
  P.out_f32 = (a.out_dtype == kF32);
  int rc;
  if (plan.kind == 0) rc = a.D == 128 ? launch_stream<128>(P, plan, a.B, a.Hkv, stream) : launch_stream<64>(P, plan, a.B, a.Hkv, stream);
  else if (plan.kind == 1) rc = a.D == 128 ? launch_rows<128, 4>(P, plan, a.B, a.Hkv, stream) : launch_rows<64, 4>(P, plan, a.B, a.Hkv, stream);
  else if (plan.kind == 2) rc = launch_rows<128, 8>(P, plan, a.B, a.Hkv, stream);
  else rc = plan.wide ? launch_rows_as<128, 8, true, 2>(P, plan, a.B, a.Hkv, stream)
                      : launch_rows_as<128, 8, false, 2>(P, plan, a.B, a.Hkv, stream);
  if (rc != 0) return rc;
  if (plan.max_chunks > 1) {
    const int max_q = a.max_q > P.n_cap ? P.n_cap : a.max_q;
    dim3 grid((max_q * a.Hq + 7) / 8, a.B);
    if (a.D == 128) hipLaunchKernelGGL(attn_combine_kernel<128>, grid, dim3(256), 0, stream, P);
    else hipLaunchKernelGGL(attn_combine_kernel<64>, grid, dim3(256), 0, stream, P);
    if (hipGetLastError() != hipSuccess) return -6;
  }
  return 0;
}

}  // namespace specv
