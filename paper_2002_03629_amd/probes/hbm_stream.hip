// Measurement probe (not part of the library): what a plain streaming kernel reads and copies per second on this
// chip -- every workgroup walks contiguous 16-byte pieces of a 2 GiB buffer (the reads are summed so that they are
// not optimised away).  The figure the HBM-bound kernels are compared with next to the nominal 8 TB/s.
#include <hip/hip_runtime.h>
#include <stdio.h>
template <int UNROLL>
__global__ __launch_bounds__(256) void rd(const uint4* __restrict__ src, size_t n16, unsigned* out) {
  unsigned acc = 0;
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) out[0] = acc;
}
__global__ __launch_bounds__(256) void cp(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}
int main() {
  const size_t bytes = (size_t)2 << 30, n16 = bytes / 16;
  uint4 *src, *dst; unsigned* out;
  if (hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&dst, bytes) != hipSuccess || hipMalloc(&out, 4) != hipSuccess ||
      hipMemset(src, 1, bytes) != hipSuccess) { printf("allocation failed\n"); return 1; }
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  for (int blocks : {1024, 2048, 4096, 8192, 16384}) {
    for (int variant = 0; variant < 3; ++variant) {
      float best = 1e9;
      for (int rep = 0; rep < 4; ++rep) {
        (void)hipEventRecord(e0);
        if (variant == 0) hipLaunchKernelGGL(rd<4>, dim3(blocks), dim3(256), 0, 0, src, n16, out);
        else if (variant == 1) hipLaunchKernelGGL(rd<8>, dim3(blocks), dim3(256), 0, 0, src, n16, out);
        else hipLaunchKernelGGL(cp, dim3(blocks), dim3(256), 0, 0, src, dst, n16);
        (void)hipEventRecord(e1);
        (void)hipEventSynchronize(e1);
        float ms = 0;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (rep && ms < best) best = ms;
      }
      printf("%s blocks %5d: %.3f ms  %.2f TB/s %s\n", variant == 0 ? "read x4 " : variant == 1 ? "read x8 " : "copy    ", blocks, best,
             bytes / best / 1e9 * (variant == 2 ? 2 : 1), variant == 2 ? "(read + write)" : "");
    }
  }
  return 0;
}
