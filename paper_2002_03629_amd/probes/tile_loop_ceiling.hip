// Measurement probe (not part of the library): what the main loop of the 256 x 256 tile kernel can reach on this chip.
// Each workgroup (4 waves, one per SIMD, 16 accumulator tiles = 256 registers per lane) runs the loop of
// masked_layer_big_kernel with nothing around it, in three stages of completeness:
//   mode 0: the MFMAs alone, operands already in registers;
//   mode 1: + the fragment reads from LDS (8 x ds_read_b128 per 16 MFMAs, one sub-step ahead);
//   mode 2: + the LDS-bound copies of the next operands from an L2-resident window and the barrier per half chunk.
// Operand data: all zeros, or dense random bf16 values -- the matrix cores' clock is power-limited, so the rate
// depends on how many bits toggle.  Prints ns per MFMA per SIMD and the chip-wide TFLOP/s.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
__device__ __forceinline__ void load_to_lds16(const void* src, uint32_t lds_byte_address) {
  uint32_t saved_m0;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0) : "v"(src), "s"(lds_byte_address) : "memory");
}
constexpr int STAGE = 2048;   // uint4 per stage (32 KB)
template <int MODE>   // 0: mfma only, 1: + lds reads, 2: + dma + barrier
__global__ __launch_bounds__(256, 1) void k(const uint4* src, size_t src_n, float* out, int halves) {
  __shared__ uint4 ring[4 * STAGE];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  for (int i = tid; i < 4 * STAGE; i += 256) ring[i] = src[(blockIdx.x * 977 + i) % src_n];
  __syncthreads();
  f32x16 acc[4][4];
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  uint4 fa0[4], fb0[4], fa1[4], fb1[4];
  auto rd = [&](const uint4* cur, int sl, uint4 (&fa)[4], uint4 (&fb)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = cur[(wm * 4 + i) * 128 + sl * 64 + lane];
#pragma unroll
    for (int j = 0; j < 4; ++j) fb[j] = cur[(8 + wn * 4 + j) * 128 + sl * 64 + lane];
  };
  auto mul = [&](const uint4 (&fa)[4], const uint4 (&fb)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[j]), __builtin_bit_cast(bf16x8, fa[i]), acc[i][j], 0, 0, 0);
  };
  const uint4* g = src + tid;   // one 1 MB window shared by all workgroups: L2 hits
  auto dma = [&](int hc, uint4* dst) {
    const uint32_t d = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)(dst + wave * 64);
#pragma unroll
    for (int q = 0; q < 8; ++q) load_to_lds16(g + ((size_t)(hc * 8 + q) * 256) % 65536, d + q * 256 * 16);
  };
  rd(ring, 0, fa0, fb0);
  rd(ring, 1, fa1, fb1);
  if (MODE == 2) for (int hc = 0; hc < 4; ++hc) dma(hc, ring + hc * STAGE);
  for (int hc = 0; hc < halves; ++hc) {
    uint4* cur = ring + (hc & 3) * STAGE;
    const uint4* next = ring + ((hc + 1) & 3) * STAGE;
    if (MODE >= 1) rd(cur, 1, fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    mul(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    if (MODE == 2) {
      asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
      dma(hc + 4, cur);
    }
    if (MODE >= 1) rd(next, 0, fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    mul(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  float s = 0;
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
int main() {
  const size_t src_n = (size_t)1 << 20;   // 16 MB of operands
  float* out;
  uint4* src;
  if (hipMalloc(&out, 4096 * 256 * 4) != hipSuccess || hipMalloc(&src, src_n * 16) != hipSuccess) { printf("hipMalloc failed\n"); return 1; }
  uint16_t* h = (uint16_t*)malloc(src_n * 16);
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  for (int mode_data = 0; mode_data < 2; ++mode_data) {
    srand(1);
    for (size_t i = 0; i < src_n * 8; ++i) {
      float f = mode_data == 0 ? 0.f : (float)((rand() % 2001) - 1000) / 400.0f;
      uint32_t u; memcpy(&u, &f, 4); h[i] = (uint16_t)(u >> 16);
    }
    if (hipMemcpy(src, h, src_n * 16, hipMemcpyHostToDevice) != hipSuccess) { printf("hipMemcpy failed\n"); return 1; }
    for (int mode = 0; mode < 3; ++mode) for (int blocks : {256, 1024}) {
      const int halves = 256;
      float best = 1e9;
      for (int rep = 0; rep < 4; ++rep) {
        (void)hipEventRecord(e0);
        if (mode == 0) hipLaunchKernelGGL(k<0>, dim3(blocks), dim3(256), 0, 0, src, src_n, out, halves);
        if (mode == 1) hipLaunchKernelGGL(k<1>, dim3(blocks), dim3(256), 0, 0, src, src_n, out, halves);
        if (mode == 2) hipLaunchKernelGGL(k<2>, dim3(blocks), dim3(256), 0, 0, src, src_n, out, halves);
        (void)hipEventRecord(e1);
        (void)hipEventSynchronize(e1);
        float ms = 0;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (rep > 0 && ms < best) best = ms;
      }
      printf("data %s mode %d (0 mfma, 1 +lds, 2 +dma+barrier) blocks %4d: %.3f ms, %.2f ns per MFMA per SIMD, %.0f TFLOP/s\n",
             mode_data ? "random" : "zeros ", mode, blocks, best, best * 1e6 / (halves * 32.0) / (blocks / 256),
             (double)blocks * 4 * halves * 32 * 32768 / best / 1e9);
      fflush(stdout);
    }
  }
  return 0;
}
