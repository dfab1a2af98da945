// Read-only streaming bandwidth probe: what a plain kernel reaches on this GPU, as context for
// the roofline fractions reported by bench.py (the nominal HBM3E peak is 8 TB/s).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ p, size_t n16, unsigned* out, int unroll_dummy) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t stride = (size_t)gridDim.x * 256;
  unsigned acc = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) { uint4 a = p[i]; acc ^= a.x ^ a.y ^ a.z ^ a.w; }
  if (acc == 0x12345678u) out[0] = acc;
}
// contiguous-per-block variant: each block reads a contiguous 64 KB run, 8 loads in flight per thread
__global__ __launch_bounds__(256) void read_block_kernel(const uint4* __restrict__ p, size_t n16, unsigned* out) {
  const size_t per_block = 4096;  // uint4 per block = 64 KB
  unsigned acc = 0;
  for (size_t base = (size_t)blockIdx.x * per_block; base < n16; base += (size_t)gridDim.x * per_block) {
    uint4 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = p[base + j * 256 + threadIdx.x];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  if (acc == 0x12345678u) out[0] = acc;
}
int main() {
  size_t bytes = (size_t)2 << 30; size_t n16 = bytes / 16;
  uint4* p; unsigned* o;
  if (hipMalloc(&p, bytes) != hipSuccess || hipMalloc(&o, 4) != hipSuccess || hipMemset(p, 1, bytes) != hipSuccess) return 1;
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  for (int grid : {1024, 2048, 4096, 8192, 16384}) {
    for (int variant = 0; variant < 2; ++variant) {
      for (int w = 0; w < 3; ++w) { if (variant == 0) read_kernel<<<grid, 256>>>(p, n16, o, 0); else read_block_kernel<<<grid, 256>>>(p, n16, o); }
      hipEventRecord(e0);
      const int it = 10;
      for (int w = 0; w < it; ++w) { if (variant == 0) read_kernel<<<grid, 256>>>(p, n16, o, 0); else read_block_kernel<<<grid, 256>>>(p, n16, o); }
      hipEventRecord(e1); hipEventSynchronize(e1);
      float ms; hipEventElapsedTime(&ms, e0, e1);
      printf("variant %d grid %5d: %.1f us/iter  %.0f GB/s\n", variant, grid, ms / it * 1e3, bytes / (ms / it * 1e-3) / 1e9);
    }
  }
  // small buffer (270 MB) one-shot rotation of 4 regions
  size_t small = (size_t)270 << 20;
  for (int it = 0; it < 8; ++it) {
    hipEventRecord(e0);
    read_block_kernel<<<4096, 256>>>(p + (it % 4) * (small / 16), small / 16, o);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    printf("270MB region %d: %.1f us  %.0f GB/s\n", it % 4, ms * 1e3, small / (ms * 1e-3) / 1e9);
  }
  return 0;
}
