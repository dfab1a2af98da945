// Device helpers shared by the gfx950 kernels of the verification library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specv {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr double kLn2 = 0.6931471805599453;

// dtype codes of the C ABI (spec_dtype)
constexpr int kBF16 = 0;
constexpr int kF32 = 1;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// 2^x through the hardware transcendental unit.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// One logit of a row-major [rows, V] matrix of either dtype, as fp32 (exact for bf16).
__device__ __forceinline__ float load_logit(const void* base, int dtype, int64_t idx) {
  if (dtype == kBF16) return bf16_bits_to_float(static_cast<const uint16_t*>(base)[idx]);
  return static_cast<const float*>(base)[idx];
}

// Eight consecutive logits of one row starting at element e0; positions >= V read as -inf.
// VEC: the row start and e0 are 16-byte aligned (V % 8 == 0 for bf16, V % 4 == 0 for fp32).
template <bool VEC>
__device__ __forceinline__ void load8(const void* base, int dtype, int64_t row_off, int e0, int V,
                                      float (&x)[8]) {
  if (dtype == kBF16) {
    const uint16_t* p = static_cast<const uint16_t*>(base) + row_off;
    if (VEC && e0 + 8 <= V) {
      const uint4 w = *reinterpret_cast<const uint4*>(p + e0);
      x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
      x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = (e0 + j < V) ? bf16_bits_to_float(p[e0 + j]) : -INFINITY;
    }
  } else {
    const float* p = static_cast<const float*>(base) + row_off;
    if (VEC && e0 + 8 <= V) {
      const float4 a = *reinterpret_cast<const float4*>(p + e0);
      const float4 b = *reinterpret_cast<const float4*>(p + e0 + 4);
      x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = (e0 + j < V) ? p[e0 + j] : -INFINITY;
    }
  }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Per-(row, segment) softmax statistics written by the row-statistics kernel:
// m = largest logit of the segment (raw logit units, -inf if the segment is empty),
// z = sum over the segment of 2^((l - m) * c), c = log2(e)/T.
struct __align__(16) SegStat {
  float m;
  float pad;
  double z;
};

}  // namespace specv
