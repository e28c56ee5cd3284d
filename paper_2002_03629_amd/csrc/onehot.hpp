// First hidden layer of a categorical model whose symbols enter as one-hot vectors (gfx950 only).
//
// With one-hot input the first masked layer is no matrix product: unit j's pre-activation is
//     b_j + sum over the positions t unit j may see of W0[j, t*C + x_t],
// one weight per visible position.  The weights are stored as [D][C][pitch] rows (units in degree order, zero
// where unit j may not see position t: a prefix of the row), so a sample's first layer is the sum of D rows
// picked by its symbols: a gather bound by HBM/L2 bandwidth.  A workgroup owns one sample and ONEHOT_UNITS
// consecutive units; a lane owns 8 units (16 bytes of bf16 per row); the sum order is fixed (see the kernel).
// Rows whose visible part starts behind the lane's units are skipped.
#pragma once

#include "resident.hpp"

namespace jm {

constexpr int ONEHOT_WAVES = 8;
constexpr int ONEHOT_THREADS = 64 * ONEHOT_WAVES;
constexpr int ONEHOT_UPT = 8;                     // units per lane: 16 bytes of bf16 per row
constexpr int ONEHOT_UNITS = 64 * ONEHOT_UPT;     // units per workgroup
constexpr int ONEHOT_DEPTH = 16;                  // rows a wave has in flight per lane

struct OnehotArgs {
  const void* Wg;        // [D][C][pitch] of T
  const float* bias;     // [pitch]
  const uint8_t* x;      // symbols [N, D]
  const int* rows;       // active-sample list or NULL (identity)
  const int* n_rows_ptr; // device count or NULL
  int n_rows;
  const int* cnt_lt;     // cnt_lt[t] = units of degree < t: the units that may see position t (0-based) start at cnt_lt[t + 1]
  int D, C, pitch;
  int t_end;             // positions [0, t_end) are read
  int unit_begin, unit_end;   // units [unit_begin, unit_end) are written (multiples of 32)
  void* out;             // activations, fragment-major with out_chunks chunks
  int out_chunks;
};

// what a lane reads instead of a row none of whose units it may see (a branch around the load would make every
// load wait for the one before it)
__device__ __align__(32) const float g_onehot_zeros[ONEHOT_UPT] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

// acc += the lane's 8 units of one weight row
template <typename T> __device__ __forceinline__ void add_row8(const T* p, float (&acc)[ONEHOT_UPT]);
template <> __device__ __forceinline__ void add_row8<bf16_t>(const bf16_t* p, float (&acc)[ONEHOT_UPT]) {
  const uint4 u = *(const uint4*)p;
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc[2 * i] += __uint_as_float(w[i] << 16);
    acc[2 * i + 1] += __uint_as_float(w[i] & 0xffff0000u);
  }
}
template <> __device__ __forceinline__ void add_row8<float>(const float* p, float (&acc)[ONEHOT_UPT]) {
  const float4 v0 = *(const float4*)p, v1 = *(const float4*)(p + 4);
  acc[0] += v0.x; acc[1] += v0.y; acc[2] += v0.z; acc[3] += v0.w;
  acc[4] += v1.x; acc[5] += v1.y; acc[6] += v1.z; acc[7] += v1.w;
}

// A workgroup owns one sample and ONEHOT_UNITS consecutive units; its waves take the positions in interleaved
// groups of ONEHOT_DEPTH (each wave adds its rows in position order, then the waves' partial sums are added in
// wave order: a fixed order), so that 16 waves per CU keep enough rows in flight to cover the memory latency.
template <typename T>
__global__ __launch_bounds__(ONEHOT_THREADS) void onehot_first_layer_kernel(OnehotArgs a) {
  __shared__ uint8_t xs[4096];
  __shared__ int first_s[4096];      // per staged position: first unit that may see it
  __shared__ float part_s[ONEHOT_WAVES][ONEHOT_UNITS];
  const int n_rows = a.n_rows_ptr ? *a.n_rows_ptr : a.n_rows;
  if ((int)blockIdx.y >= n_rows) return;
  const int sample = a.rows ? a.rows[blockIdx.y] : (int)blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u0 = a.unit_begin + blockIdx.x * ONEHOT_UNITS + ONEHOT_UPT * lane;
  const bool mine = u0 < a.unit_end;           // (unit_end is a multiple of 32, u0 of 8: all 8 units or none)
  const T* Wg = (const T*)a.Wg;
  float acc[ONEHOT_UPT];
#pragma unroll
  for (int e = 0; e < ONEHOT_UPT; ++e) acc[e] = 0.f;
  // positions are taken in slabs of 4096 symbols staged in LDS
  for (int s0 = 0; s0 < a.t_end; s0 += 4096) {
    const int s1 = min(a.t_end, s0 + 4096);
    __syncthreads();
    for (int i = threadIdx.x; i < s1 - s0; i += ONEHOT_THREADS) {
      xs[i] = a.x[(size_t)sample * a.D + s0 + i];
      first_s[i] = a.cnt_lt[s0 + i + 1];
    }
    __syncthreads();
    if (mine) {
      for (int t = s0 + wave * ONEHOT_DEPTH; t < s1; t += ONEHOT_WAVES * ONEHOT_DEPTH) {
        // independent loads: all rows of a group are requested before the first add
        float part[ONEHOT_DEPTH][ONEHOT_UPT];
#pragma unroll
        for (int i = 0; i < ONEHOT_DEPTH; ++i) {
          const int tt = min(t + i, s1 - 1);
          const bool on = t + i < s1 && u0 + ONEHOT_UPT - 1 >= first_s[tt - s0];      // some of these units see position tt
          const T* p = Wg + ((size_t)tt * a.C + min((int)xs[tt - s0], a.C - 1)) * a.pitch + u0;   // (a symbol >= C reads class C-1)
#pragma unroll
          for (int e = 0; e < ONEHOT_UPT; ++e) part[i][e] = 0.f;
          add_row8<T>(on ? p : (const T*)g_onehot_zeros, part[i]);
        }
#pragma unroll
        for (int i = 0; i < ONEHOT_DEPTH; ++i)
#pragma unroll
          for (int e = 0; e < ONEHOT_UPT; ++e) acc[e] += part[i][e];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < ONEHOT_UPT; ++e) part_s[wave][ONEHOT_UPT * lane + e] = acc[e];
  __syncthreads();
  if (wave == 0 && mine) {
    float v[ONEHOT_UPT];
#pragma unroll
    for (int e = 0; e < ONEHOT_UPT; ++e) {
      float s = part_s[0][ONEHOT_UPT * lane + e];
#pragma unroll
      for (int w = 1; w < ONEHOT_WAVES; ++w) s += part_s[w][ONEHOT_UPT * lane + e];
      v[e] = fmaxf(s + a.bias[u0 + e], 0.f);
    }
    const float lo[4] = {v[0], v[1], v[2], v[3]}, hi[4] = {v[4], v[5], v[6], v[7]};
    store4<T>((T*)a.out + frag_offset<T>(sample, u0, a.out_chunks), lo);
    store4<T>((T*)a.out + frag_offset<T>(sample, u0 + 4, a.out_chunks), hi);
  }
}

}  // namespace jm
