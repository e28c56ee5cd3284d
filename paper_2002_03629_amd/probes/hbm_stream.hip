// Measurement probe (not part of the library): what a plain streaming kernel reads and copies per second on this
// chip.  A 2 GiB buffer is read in 16-byte pieces per lane (the reads are summed so that they are not optimised
// away), in three ways: every workgroup striding through the whole buffer, every workgroup walking one contiguous
// piece of it, and the latter with non-temporal loads.  The figures the HBM-bound kernels are compared with next to
// the nominal 8 TB/s.
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
// PIECE: 0 = the grid strides through the buffer together, 1 = a workgroup owns a contiguous piece; NT: non-temporal loads
template <int UNROLL, int PIECE, bool NT>
__global__ __launch_bounds__(256) void rd(const u32x4* __restrict__ src, size_t n16, unsigned* out) {
  unsigned acc = 0;
  size_t i, end, stride;
  if (PIECE == 0) {
    stride = (size_t)gridDim.x * 256;
    i = (size_t)blockIdx.x * 256 + threadIdx.x;
    end = n16;
  } else {
    const size_t per = n16 / gridDim.x;
    stride = 256;
    i = per * blockIdx.x + threadIdx.x;
    end = per * (blockIdx.x + 1);
  }
  for (; i + (UNROLL - 1) * stride < end; i += UNROLL * stride) {
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = NT ? __builtin_nontemporal_load(src + i + u * stride) : src[i + u * stride];
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
  const char* names[4] = {"read, grid-strided        ", "read, piece per workgroup ", "read, piece, non-temporal ", "copy, grid-strided        "};
  for (int blocks : {2048, 8192, 32768}) {
    for (int variant = 0; variant < 4; ++variant) {
      float best = 1e9;
      for (int rep = 0; rep < 4; ++rep) {
        (void)hipEventRecord(e0);
        if (variant == 0) hipLaunchKernelGGL((rd<8, 0, false>), dim3(blocks), dim3(256), 0, 0, (const u32x4*)src, n16, out);
        else if (variant == 1) hipLaunchKernelGGL((rd<8, 1, false>), dim3(blocks), dim3(256), 0, 0, (const u32x4*)src, n16, out);
        else if (variant == 2) hipLaunchKernelGGL((rd<8, 1, true>), dim3(blocks), dim3(256), 0, 0, (const u32x4*)src, n16, out);
        else hipLaunchKernelGGL(cp, dim3(blocks), dim3(256), 0, 0, src, dst, n16);
        (void)hipEventRecord(e1);
        (void)hipEventSynchronize(e1);
        float ms = 0;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (rep && ms < best) best = ms;
      }
      printf("%s blocks %5d: %.3f ms  %.2f TB/s %s\n", names[variant], blocks, best, bytes / best / 1e9 * (variant == 3 ? 2 : 1),
             variant == 3 ? "(read + write)" : "");
    }
  }
  return 0;
}
