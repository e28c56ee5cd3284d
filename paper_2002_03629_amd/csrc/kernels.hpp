// Device code of libjacobi_made.so (gfx950 only).
//
// One Jacobi pass (the loop body of Algorithm 1) is: every hidden masked layer, then the output
// masked layer whose epilogue draws the symbols from the fixed noise (Appendix A.3) and counts,
// per sample, how many positions changed (the forward difference of Section 2.2.1 with
// tolerance 0).  A small kernel then retires unchanged samples from the active list.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jm {

typedef uint16_t bf16_t;  // storage type; arithmetic goes through float
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
  static constexpr int EPL = 32;  // elements one lane loads per K chunk (64 bytes)
  static __device__ __forceinline__ bf16_t from_f32(float f) { return f32_to_bf16(f); }
};
template <> struct Elem<float> {
  static constexpr int EPL = 16;
  static __device__ __forceinline__ float from_f32(float f) { return f; }
};

constexpr int TILE = 32;   // output tile: 32 samples x 32 units per workgroup
constexpr int WAVES = 4;   // the 4 waves of a workgroup split the K range between them

enum Epilogue { EPI_RELU = 0, EPI_LOGITS = 1, EPI_BERNOULLI = 2 };

struct LayerArgs {
  // operands: A = activations [sample, lda], W = masked weights [unit, ldw], both K-contiguous
  const void* A;
  int lda;
  const void* W;
  int ldw;
  const float* bias;     // [out_pad]
  const int* tile_kend;  // per 32-unit tile: K extent that holds non-zero (visible) weights, chunk-rounded
  int k_cap;             // additional upper limit on K (chunk-rounded)
  int tile_begin;        // first unit tile this launch covers (blockIdx.x is relative to it)
  // active samples: rows[0 .. *n_rows_ptr) are sample ids (NULL = identity, n_rows fixed)
  const int* rows;
  const int* n_rows_ptr;
  int n_rows;
  // EPI_RELU: out = activations [sample, ldo] of type T.  EPI_LOGITS: out = float [sample, ldo]
  void* out;
  int ldo;
  int n_cols;            // real (unpadded) number of units of this layer
  // EPI_BERNOULLI
  const float* noise;    // u[sample, D]
  uint8_t* x;            // [sample, D], updated in place
  void* enc;             // network input of the next pass, T [sample, ld_enc]
  int ld_enc;
  int* changed;          // per-sample count of positions whose symbol changed
  int D;
  int t_lo, t_hi;        // only positions in [t_lo, t_hi) are re-drawn
};

template <typename T>
__device__ __forceinline__ void mfma_chunk(const uint4 (&a)[4], const uint4 (&b)[4], f32x16& acc);

template <>
__device__ __forceinline__ void mfma_chunk<bf16_t>(const uint4 (&a)[4], const uint4 (&b)[4], f32x16& acc) {
#pragma unroll
  for (int s = 0; s < 4; ++s)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[s]),
                                                  __builtin_bit_cast(bf16x8, b[s]), acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mfma_chunk<float>(const uint4 (&a)[4], const uint4 (&b)[4], f32x16& acc) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[s].x), __uint_as_float(b[s].x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[s].y), __uint_as_float(b[s].y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[s].z), __uint_as_float(b[s].z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[s].w), __uint_as_float(b[s].w), acc, 0, 0, 0);
  }
}

// One masked dense layer on a 32 x 32 output tile per workgroup.
//
// Lane (r = lane % 32, h = lane / 32) of a wave owns sample row r and weight row r of the tile and
// loads 64 contiguous bytes of each per K chunk, the h-th half of the chunk.  The MFMA contracts
// lane-held K slices of A against the same slices of B, so which physical K a slot carries does
// not matter as long as both operands agree -- this keeps every global load 64 bytes wide and
// contiguous.  The four waves take K chunks round-robin and their partial tiles are summed
// through LDS in a fixed order (deterministic results).
template <typename T, int EPI>
__global__ __launch_bounds__(256) void masked_layer_kernel(LayerArgs a) {
  constexpr int EPL = Elem<T>::EPL;
  constexpr int KC = 2 * EPL;
  __shared__ float part[WAVES][TILE][TILE + 1];

  const int n_rows = a.n_rows_ptr ? *a.n_rows_ptr : a.n_rows;
  const int row0 = blockIdx.y * TILE;
  if (row0 >= n_rows) return;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int tile = a.tile_begin + blockIdx.x;
  const int col0 = tile * TILE;

  int my_row = row0 + r;
  int my_sample = my_row < n_rows ? (a.rows ? a.rows[my_row] : my_row) : 0;  // clamped rows are discarded below
  const T* Ap = (const T*)a.A + (size_t)my_sample * a.lda + h * EPL;
  const T* Wp = (const T*)a.W + (size_t)(col0 + r) * a.ldw + h * EPL;
  int k_end = a.tile_kend[tile];
  if (k_end > a.k_cap) k_end = a.k_cap;

  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  for (int kc = wave * KC; kc < k_end; kc += WAVES * KC) {
    uint4 av[4], bv[4];
    const uint4* ap = (const uint4*)(Ap + kc);
    const uint4* wp = (const uint4*)(Wp + kc);
#pragma unroll
    for (int s = 0; s < 4; ++s) { av[s] = ap[s]; bv[s] = wp[s]; }
    mfma_chunk<T>(av, bv, acc);
  }

  // acc[i] is the tile element (row = 8*(i/4) + 4*h + i%4, col = r): rows come from A = samples
#pragma unroll
  for (int i = 0; i < 16; ++i) part[wave][(i >> 2) * 8 + h * 4 + (i & 3)][r] = acc[i];
  __syncthreads();

  const int rr = threadIdx.x >> 3, c0 = (threadIdx.x & 7) * 4;
  const int out_row = row0 + rr;
  const bool row_ok = out_row < n_rows;
  const int sample = row_ok ? (a.rows ? a.rows[out_row] : out_row) : 0;
  float v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    v[j] = ((part[0][rr][c0 + j] + part[1][rr][c0 + j]) + (part[2][rr][c0 + j] + part[3][rr][c0 + j])) +
           a.bias[col0 + c0 + j];

  if (EPI == EPI_RELU) {
    if (row_ok) {
      T* o = (T*)a.out + (size_t)sample * a.ldo + col0 + c0;
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = Elem<T>::from_f32(fmaxf(v[j], 0.f));
    }
  } else if (EPI == EPI_LOGITS) {
    if (row_ok) {
      float* o = (float*)a.out + (size_t)sample * a.ldo;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (col0 + c0 + j < a.n_cols) o[col0 + c0 + j] = v[j];
    }
  } else {  // EPI_BERNOULLI: x_t = 1 iff u_t < sigmoid(z_t); count changes per sample
    int cnt = 0;
    if (row_ok) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int t = col0 + c0 + j;
        if (t >= a.t_lo && t < a.t_hi) {
          const size_t idx = (size_t)sample * a.D + t;
          const float p = 1.0f / (1.0f + expf(-v[j]));
          const uint8_t xn = a.noise[idx] < p ? 1 : 0;
          cnt += (xn != a.x[idx]);
          a.x[idx] = xn;
          ((T*)a.enc)[(size_t)sample * a.ld_enc + t] = Elem<T>::from_f32((float)xn);
        }
      }
    }
    cnt += __shfl_xor(cnt, 1);
    cnt += __shfl_xor(cnt, 2);
    cnt += __shfl_xor(cnt, 4);
    if ((threadIdx.x & 7) == 0 && cnt > 0) atomicAdd(&a.changed[sample], cnt);
  }
}

// Gumbel-max draw for categorical positions from logits held in memory:
// x[n, t] = argmax_c (z[n, t, c] + g[n, t, c]), lowest c on ties.  One wave per (row, t).
template <typename T>
__global__ __launch_bounds__(256) void gumbel_argmax_kernel(const float* __restrict__ z, int ldz,
                                                            const float* __restrict__ g, uint8_t* x, T* enc,
                                                            int ld_enc, int* changed, const int* rows,
                                                            const int* n_rows_ptr, int n_rows_fixed, int D, int C,
                                                            int t_lo, int t_hi) {
  const int n_rows = n_rows_ptr ? *n_rows_ptr : n_rows_fixed;
  const int lane = threadIdx.x & 63;
  const int wave_global = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int span = t_hi - t_lo;
  const int row = wave_global / span, t = t_lo + wave_global % span;
  if (row >= n_rows) return;
  const int sample = rows ? rows[row] : row;
  const float* zp = z + (size_t)sample * ldz + (size_t)t * C;
  const float* gp = g + ((size_t)sample * D + t) * C;
  float best = -INFINITY;
  int best_c = 0x7fffffff;
  for (int c = lane; c < C; c += 64) {
    const float s = zp[c] + gp[c];
    if (s > best || (s == best && c < best_c)) { best = s; best_c = c; }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ob = __shfl_xor(best, off);
    const int oc = __shfl_xor(best_c, off);
    if (ob > best || (ob == best && oc < best_c)) { best = ob; best_c = oc; }
  }
  if (lane == 0) {
    const size_t idx = (size_t)sample * D + t;
    const uint8_t xn = (uint8_t)best_c;
    if (xn != x[idx]) atomicAdd(&changed[sample], 1);
    x[idx] = xn;
    enc[(size_t)sample * ld_enc + t] = Elem<T>::from_f32(((float)xn - 128.0f) * (1.0f / 128.0f));
  }
}

// Start of a call: x = x_init (or zeros), enc = network input of x, bookkeeping cleared.
template <typename T>
__global__ void init_state_kernel(const uint8_t* x_init, uint8_t* x, T* enc, int ld_enc, int N, int D, int C) {
  const size_t total = (size_t)N * D;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int n = (int)(i / D), t = (int)(i % D);
    const uint8_t v = x_init ? x_init[i] : 0;
    if (x) x[i] = v;
    const float e = (C == 1) ? (float)v : ((float)v - 128.0f) * (1.0f / 128.0f);
    enc[(size_t)n * ld_enc + t] = Elem<T>::from_f32(e);
  }
}

__global__ void reset_rows_kernel(int* rows, int* n_rows, int N, int* changed, int* iters, int* flags) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < N) {
    rows[i] = i;
    changed[i] = 0;
    if (iters) iters[i] = 0;
  }
  if (i == 0) {
    *n_rows = N;
    if (flags) *flags = 0;
  }
}

// After a pass: every active sample took one more pass; the ones whose block changed stay active
// (order preserved), unless this was the last allowed pass.  Single workgroup of 256 threads.
__global__ __launch_bounds__(256) void retire_kernel(const int* rows_in, const int* n_in, int* rows_out, int* n_out,
                                                     int* changed, int* iters, int last_pass, int flag_unconverged,
                                                     int* flags) {
  __shared__ int wave_total[4];
  __shared__ int base_s;
  const int n_rows = *n_in;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) base_s = 0;
  __syncthreads();
  for (int start = 0; start < n_rows; start += 256) {
    const int rix = start + threadIdx.x;
    int sample = -1;
    bool keep = false;
    if (rix < n_rows) {
      sample = rows_in[rix];
      const int c = changed[sample];
      changed[sample] = 0;
      iters[sample] += 1;
      keep = (c > 0) && !last_pass;
      if (c > 0 && last_pass && flag_unconverged) atomicOr(flags, 1);
    }
    const unsigned long long mask = __ballot(keep);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_total[wave] = __popcll(mask);
    __syncthreads();
    int off = base_s;
    for (int w = 0; w < wave; ++w) off += wave_total[w];
    if (keep) rows_out[off + before] = sample;
    __syncthreads();
    if (threadIdx.x == 0) base_s += wave_total[0] + wave_total[1] + wave_total[2] + wave_total[3];
    __syncthreads();
  }
  if (threadIdx.x == 0) *n_out = base_s;
}

}  // namespace jm
