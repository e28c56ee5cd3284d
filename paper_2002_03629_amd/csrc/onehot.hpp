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
constexpr int ONEHOT_SUB = 1;                     // sub-blocks of 512 units per workgroup (2: same time, 4: slower)
constexpr int ONEHOT_UNITS = 512 * ONEHOT_SUB;    // units per workgroup
constexpr int ONEHOT_DEPTH = 8;                    // rows per register set: a wave has one or two sets in flight

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
__device__ __align__(32) const float g_onehot_zeros[8] = {};

// The lane's 8 units of one weight row as loaded (16 bytes of bf16, 32 of fp32; non-temporal loads), and their
// addition to the lane's sums.
template <typename T> struct RowPiece;
template <> struct RowPiece<bf16_t> { uint4 a; };
template <> struct RowPiece<float> { uint4 a, b; };
__device__ __forceinline__ RowPiece<bf16_t> load_row8(const bf16_t* p) { return {load_stream16((const uint4*)p)}; }
__device__ __forceinline__ RowPiece<float> load_row8(const float* p) {
  return {load_stream16((const uint4*)p), load_stream16((const uint4*)p + 1)};
}
__device__ __forceinline__ void add_row8(const RowPiece<bf16_t>& r, float (&acc)[8]) {
  const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc[2 * i] += __uint_as_float(w[i] << 16);
    acc[2 * i + 1] += __uint_as_float(w[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void add_row8(const RowPiece<float>& r, float (&acc)[8]) {
  acc[0] += __uint_as_float(r.a.x); acc[1] += __uint_as_float(r.a.y); acc[2] += __uint_as_float(r.a.z); acc[3] += __uint_as_float(r.a.w);
  acc[4] += __uint_as_float(r.b.x); acc[5] += __uint_as_float(r.b.y); acc[6] += __uint_as_float(r.b.z); acc[7] += __uint_as_float(r.b.w);
}

// A workgroup owns one sample and ONEHOT_UNITS consecutive units at a time; its waves take the positions in
// interleaved groups of ONEHOT_DEPTH (each wave adds its rows in position order, then the waves' partial sums are
// added in wave order: a fixed order), so that the waves of a compute unit keep enough rows in flight to cover the
// memory latency.  A lane owns 8 units in each of the ONEHOT_SUB sub-blocks of 512 units, so one load instruction of a
// wave takes 1 KB of a row in whole cache lines, with the non-temporal hint: nothing of the 800 MB is worth keeping,
// and without it the stream pushes the next layers' weights out of the caches (cfg4 with one-hot input: this launch
// 52.8 -> 47.5 us, the second hidden layer 11.2 -> 9.8 us, the output layer 143.5 -> 140.9 us).
// Units are laid out by degree, so the positions a chunk of units can see are a PREFIX of the positions, longer the
// higher the chunk: a chunk only walks its prefix (requests for rows nobody of the chunk sees would occupy the places
// of real ones), and a workgroup takes TWO chunks, c from the end and c from the start, one after the other, so that
// every workgroup walks about the same number of rows.
template <typename T>
__global__ __launch_bounds__(ONEHOT_THREADS) void onehot_first_layer_kernel(OnehotArgs a) {
  __shared__ uint8_t xs[4096];
  __shared__ int first_s[4096];      // per staged position: first unit that may see it
  __shared__ float part_s[ONEHOT_WAVES][ONEHOT_UNITS];
  __shared__ int visible_s;
  const int n_rows = a.n_rows_ptr ? *a.n_rows_ptr : a.n_rows;
  if ((int)blockIdx.y >= n_rows) return;
  const int sample = a.rows ? a.rows[blockIdx.y] : (int)blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunks = (a.unit_end - a.unit_begin + ONEHOT_UNITS - 1) / ONEHOT_UNITS;
  const T* Wg = (const T*)a.Wg;
  const bool one_slab = a.t_end <= 4096;         // (then the symbols are staged once, for both chunks)
  for (int part = 0; part < 2; ++part) {
    const int chunk = part == 0 ? chunks - 1 - (int)blockIdx.x : (int)blockIdx.x;
    if (part == 1 && chunk >= chunks - 1 - (int)blockIdx.x) break;   // (an odd number of chunks: the middle one is part 0's)
    const int u0 = a.unit_begin + chunk * ONEHOT_UNITS + 8 * lane;   // sub-block b: units u0 + 512 b .. + 7
    // (unit_end is a multiple of 32, the sub-blocks' first units of 8: all 8 units of a sub-block or none)
    const int u_last = min(a.unit_begin + (chunk + 1) * ONEHOT_UNITS, a.unit_end) - 1;
    float acc[ONEHOT_SUB][8];
#pragma unroll
    for (int b = 0; b < ONEHOT_SUB; ++b)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;
    // positions are taken in slabs of 4096 symbols staged in LDS
    for (int s0 = 0; s0 < a.t_end; s0 += 4096) {
      const int s1 = min(a.t_end, s0 + 4096);
      __syncthreads();                           // (the slab and the counter are free)
      if (part == 0 || !one_slab)
        for (int i = threadIdx.x; i < s1 - s0; i += ONEHOT_THREADS) {
          xs[i] = a.x[(size_t)sample * a.D + s0 + i];
          first_s[i] = a.cnt_lt[s0 + i + 1];
        }
      if (threadIdx.x == 0) visible_s = 0;
      __syncthreads();
      // the slab's positions that some unit of the chunk sees: a prefix (first_s ascends)
      int mine_visible = 0;
      for (int i = threadIdx.x; i < s1 - s0; i += ONEHOT_THREADS) mine_visible += first_s[i] <= u_last ? 1 : 0;
      if (mine_visible) atomicAdd(&visible_s, mine_visible);
      __syncthreads();
      const int sv = s0 + visible_s;             // positions [s0, sv) are walked
      // Two sets of ONEHOT_DEPTH rows: while one set's rows are added, the other set's are on their way (a wave that
      // requests, waits and adds in turn has nothing in flight while it adds).  Rows are added in position order.
      RowPiece<T> raw[2][ONEHOT_DEPTH][ONEHOT_SUB];
      auto request = [&](int t, auto SET) {
        constexpr int set = decltype(SET)::value;
#pragma unroll
        for (int i = 0; i < ONEHOT_DEPTH; ++i) {
          const int tt = min(t + i, sv - 1);
          const int first = t + i < sv ? first_s[tt - s0] : 0x7fffffff;
          const T* p = Wg + ((size_t)tt * a.C + min((int)xs[tt - s0], a.C - 1)) * a.pitch + u0;   // (a symbol >= C reads class C-1)
#pragma unroll
          for (int b = 0; b < ONEHOT_SUB; ++b) {
            const int ub = u0 + 512 * b;
            const bool on = ub < a.unit_end && ub + 7 >= first;            // some of these units see position tt
            // (a lane that sees nothing reads zeros instead of branching around the load: a branch would make every
            // load wait for the one before it)
            raw[set][i][b] = load_row8(on ? p + 512 * b : (const T*)g_onehot_zeros);
          }
        }
      };
      auto add = [&](auto SET) {
        constexpr int set = decltype(SET)::value;
#pragma unroll
        for (int i = 0; i < ONEHOT_DEPTH; ++i)
#pragma unroll
          for (int b = 0; b < ONEHOT_SUB; ++b) add_row8(raw[set][i][b], acc[b]);
      };
      const std::integral_constant<int, 0> set0;
      const std::integral_constant<int, 1> set1;
      const int step = ONEHOT_WAVES * ONEHOT_DEPTH;
      int t = s0 + wave * ONEHOT_DEPTH;
      if (t < sv) request(t, set0);
      for (; t < sv; t += 2 * step) {
        if (t + step < sv) request(t + step, set1);
        __builtin_amdgcn_sched_barrier(0);
        add(set0);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 * step < sv) request(t + 2 * step, set0);
        __builtin_amdgcn_sched_barrier(0);
        if (t + step < sv) add(set1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (part == 1) __syncthreads();              // (part 0's partial sums have been read)
#pragma unroll
    for (int b = 0; b < ONEHOT_SUB; ++b)
#pragma unroll
      for (int e = 0; e < 8; ++e) part_s[wave][512 * b + 8 * lane + e] = acc[b][e];
    __syncthreads();
    if (wave < ONEHOT_SUB && u0 + 512 * wave < a.unit_end) {               // wave b finishes sub-block b
      const int ub = u0 + 512 * wave;
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float s = part_s[0][512 * wave + 8 * lane + e];
#pragma unroll
        for (int w = 1; w < ONEHOT_WAVES; ++w) s += part_s[w][512 * wave + 8 * lane + e];
        v[e] = fmaxf(s + a.bias[ub + e], 0.f);
      }
      const float lo[4] = {v[0], v[1], v[2], v[3]}, hi[4] = {v[4], v[5], v[6], v[7]};
      store4<T>((T*)a.out + frag_offset<T>(sample, ub, a.out_chunks), lo);
      store4<T>((T*)a.out + frag_offset<T>(sample, ub + 4, a.out_chunks), hi);
    }
  }
}

}  // namespace jm
