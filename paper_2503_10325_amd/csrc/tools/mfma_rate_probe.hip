// Stand-alone probe (context for the matrix-core roofline numbers): the dense bf16 rate the chip
// sustains when every wave issues independent v_mfma_f32_32x32x16_bf16 from registers (no memory
// traffic), and the shader clock it holds meanwhile (shader cycles against the 100 MHz wall clock).
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
__global__ __launch_bounds__(256) void k(float* out, int iters, long long* clk) {
  f32x16 acc[8];
  for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f + i); b[i] = (__bf16)(blockIdx.x * 0.002f - i); }
  long long t0 = clock64(); long long w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  long long t1 = clock64(); long long w1 = wall_clock64();
  float s = 0.f;
  for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { clk[0] = t1 - t0; clk[1] = w1 - w0; }
}
int main() {
  float* out; long long* clk;
  hipMalloc(&out, 4096 * 256 * 4); hipMalloc(&clk, 16);
  for (int wpc = 1; wpc <= 2; ++wpc) {
    int blocks = 256 * wpc, iters = 20000;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    hipLaunchKernelGGL(k, dim3(blocks), dim3(256), 0, 0, out, 100, clk);
    hipDeviceSynchronize();
    hipEventRecord(e0);
    hipLaunchKernelGGL(k, dim3(blocks), dim3(256), 0, 0, out, iters, clk);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    long long h[2]; hipMemcpy(h, clk, 16, hipMemcpyDeviceToHost);
    double flop = (double)blocks * 4 * iters * 8 * 32768.0;
    printf("workgroups/CU %d: %.3f ms, %.0f TFLOP/s; shader clocks %lld, wall ticks %lld (100 MHz) -> %.0f MHz\n", wpc, ms,
           flop / ms / 1e9, h[0], h[1], (double)h[0] / ((double)h[1] / 100.0));
  }
  return 0;
}
