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
#ifndef JM_NW
#define JM_NW 8
#endif
#ifndef JM_PD
#define JM_PD 4
#endif
constexpr int NW = JM_NW;  // waves per workgroup; they split the K range between them
constexpr int PD = JM_PD;  // K chunks a wave keeps in flight (all their loads are issued before the first MFMA)
constexpr int XCDS = 8;    // workgroup i is dispatched to XCD i % 8; each XCD has its own L2

enum Epilogue { EPI_RELU = 0, EPI_LOGITS = 1, EPI_BERNOULLI = 2 };

// What the last workgroup of a pass's final kernel does once every workgroup is done: retire the
// samples that did not change and tell the host how many are left (see retire_tail).
struct RetireArgs {
  const int* rows_in;
  const int* n_in;
  int* rows_out;
  int* n_out;
  int* changed;          // per-sample changed-position counters of this pass (cleared here)
  int* iters;            // per-sample pass counters
  int* flags;            // bit 0: some sample was still changing after the last allowed pass
  int* done_ctr;         // workgroups finished so far in this kernel (cleared here)
  int* host_slot;        // device-visible pinned host word receiving the new active count
  int last_pass;
  int flag_unconverged;
  int enabled;
};

struct LayerArgs {
  // operands: A = activations [sample, lda], W = masked weights [unit, ldw], both K-contiguous
  const void* A;
  int lda;
  const void* W;
  int ldw;
  const float* bias;     // [out_pad]
  const int* tile_kend;  // per 32-unit tile: K extent that holds non-zero (visible) weights, chunk-rounded
  int k_cap;             // additional upper limit on K (chunk-rounded)
  int tile_begin;        // first unit tile this launch covers
  int n_launch_tiles;    // unit tiles this launch covers
  int row_tiles;         // sample tiles this launch covers (upper bound; tiles beyond n_rows idle)
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
  RetireArgs retire;
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

// Stop test and compaction (the forward-difference test of Algorithm 1 with tolerance 0, per
// sample): every active sample took one more pass; those whose symbols changed stay active, in
// order, unless this was the last allowed pass.  Runs in ONE workgroup, after all others finished.
__device__ __forceinline__ void retire_tail(const RetireArgs& r) {
  __shared__ int wave_total[NW];
  __shared__ int base_s;
  const int nthreads = blockDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = nthreads >> 6;
  const int n_rows = *r.n_in;
  if (threadIdx.x == 0) base_s = 0;
  __syncthreads();
  for (int start = 0; start < n_rows; start += nthreads) {
    const int rix = start + threadIdx.x;
    int sample = -1;
    bool keep = false;
    if (rix < n_rows) {
      sample = r.rows_in[rix];
      // counters were built with device-scope atomics by workgroups on other XCDs: read them the same way
      const int c = __hip_atomic_load(&r.changed[sample], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      r.changed[sample] = 0;
      r.iters[sample] += 1;
      keep = (c > 0) && !r.last_pass;
      if (c > 0 && r.last_pass && r.flag_unconverged) atomicOr(r.flags, 1);
    }
    const unsigned long long mask = __ballot(keep);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_total[wave] = __popcll(mask);
    __syncthreads();
    int off = base_s;
    for (int w = 0; w < wave; ++w) off += wave_total[w];
    if (keep) r.rows_out[off + before] = sample;
    __syncthreads();
    if (threadIdx.x == 0) {
      int tot = 0;
      for (int w = 0; w < nwaves; ++w) tot += wave_total[w];
      base_s += tot;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *r.n_out = base_s;
    *r.done_ctr = 0;
    // the host reads nothing but this word before it synchronises the stream: no release needed
    __hip_atomic_store(r.host_slot, base_s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

// Add to a per-sample changed counter and wait until the atomic has been performed (its old value
// came back), so that a later atomic on done_ctr is ordered after it without a memory fence.
__device__ __forceinline__ void count_changed(int* counter, int cnt) {
  const int old = __hip_atomic_fetch_add(counter, cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("" ::"v"(old));
}

// Every workgroup calls this at the end of the pass's final kernel; exactly one of them (the last to
// arrive) runs the retire step.  The only data the retire step reads from other workgroups are the
// changed counters; they are written and read with device-scope atomics, and every workgroup has seen
// its own counter atomics return before it bumps done_ctr, so no cache write-back is needed here.
__device__ __forceinline__ void finish_pass(const RetireArgs& r, int total_workgroups) {
  __shared__ int is_last_s;
  __syncthreads();
  if (threadIdx.x == 0)
    is_last_s = (__hip_atomic_fetch_add(r.done_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                 total_workgroups - 1);
  __syncthreads();
  if (is_last_s) retire_tail(r);
}

// One masked dense layer on a 32 x 32 output tile per workgroup.
//
// Lane (r = lane % 32, h = lane / 32) of a wave owns sample row r and weight row r of the tile and
// loads 64 contiguous bytes of each per K chunk, the h-th half of the chunk.  The MFMA contracts
// lane-held K slices of A against the same slices of B, so which physical K a slot carries does
// not matter as long as both operands agree -- this keeps every global load 64 bytes wide and
// contiguous.  At batch sizes around 100 a tile's whole K range is only a few hundred KB, so the
// kernel is bound by memory latency and by the rate at which waves can be dispatched, not by
// bandwidth or MFMA rate: a workgroup has only 4 waves, they take K chunks round-robin, and each
// wave issues the loads of up to PD chunks before its first MFMA, which puts (nearly) the entire
// tile in flight at once.  Partial tiles are summed through LDS in a fixed
// order (deterministic results).  Workgroups are numbered so that the sample tiles sharing a
// weight tile run on the same XCD and hit that XCD's L2.
template <typename T, int EPI>
__global__ __launch_bounds__(NW * 64) void masked_layer_kernel(LayerArgs a) {
  constexpr int EPL = Elem<T>::EPL;
  constexpr int KC = 2 * EPL;
  constexpr int EPT = TILE * TILE / (NW * 64);   // tile elements each thread finishes in the epilogue
  __shared__ float part[NW][TILE][TILE + 1];

  const int xcd = blockIdx.x % XCDS, slot = blockIdx.x / XCDS;
  const int row0 = (slot % a.row_tiles) * TILE;
  const int rel_tile = (slot / a.row_tiles) * XCDS + xcd;
  if (rel_tile < a.n_launch_tiles) {   // (uniform per workgroup)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int tile = a.tile_begin + rel_tile;
    const int col0 = tile * TILE;
    const int cc = threadIdx.x & 31, col = col0 + cc;

    // Everything that does not depend on other loads is requested up front, so the kernel is a chain of
    // only three memory round trips (bookkeeping, operands, results).  Entries of `rows` past the active
    // count are stale but valid sample ids, so they can be read before the count is known.
    const int n_rows = a.n_rows_ptr ? *a.n_rows_ptr : a.n_rows;
    const int my_sample = a.rows ? a.rows[row0 + r] : (row0 + r < a.n_rows ? row0 + r : 0);
    int k_end = a.tile_kend[tile];
    const float bias = a.bias[col];
    int e_sample[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      const int rr = (threadIdx.x >> 5) + j * (NW * 2);
      e_sample[j] = a.rows ? a.rows[row0 + rr] : (row0 + rr < a.n_rows ? row0 + rr : 0);
    }
    float e_noise[EPT];
    uint8_t e_xold[EPT];
    const bool col_live = EPI == EPI_BERNOULLI && col >= a.t_lo && col < a.t_hi;
    if (EPI == EPI_BERNOULLI) {
#pragma unroll
      for (int j = 0; j < EPT; ++j) {
        e_noise[j] = 0.f;
        e_xold[j] = 0;
        if (col_live) {
          const size_t idx = (size_t)e_sample[j] * a.D + col;
          e_noise[j] = a.noise[idx];
          e_xold[j] = a.x[idx];
        }
      }
    }

    if (row0 < n_rows) {
      const T* Ap = (const T*)a.A + (size_t)my_sample * a.lda + h * EPL;
      const T* Wp = (const T*)a.W + (size_t)(col0 + r) * a.ldw + h * EPL;
      if (k_end > a.k_cap) k_end = a.k_cap;

      f32x16 acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;

      const int n_chunks = (k_end + KC - 1) / KC;
      const int n_mine = (n_chunks - wave + NW - 1) / NW;   // chunks wave, wave + NW, ... belong to this wave
      for (int base = 0; base < n_mine; base += PD) {
        uint4 av[PD][4], bv[PD][4];
#pragma unroll
        for (int p = 0; p < PD; ++p) {
          if (base + p < n_mine) {
            const int kc = ((base + p) * NW + wave) * KC;
            const uint4* ap = (const uint4*)(Ap + kc);
            const uint4* wp = (const uint4*)(Wp + kc);
#pragma unroll
            for (int s = 0; s < 4; ++s) { av[p][s] = ap[s]; bv[p][s] = wp[s]; }
          }
        }
#pragma unroll
        for (int p = 0; p < PD; ++p)
          if (base + p < n_mine) mfma_chunk<T>(av[p], bv[p], acc);
      }

      // acc[i] is the tile element (row = 8*(i/4) + 4*h + i%4, col = r): rows come from A = samples
#pragma unroll
      for (int i = 0; i < 16; ++i) part[wave][(i >> 2) * 8 + h * 4 + (i & 3)][r] = acc[i];
      __syncthreads();

#pragma unroll
      for (int j = 0; j < EPT; ++j) {
        const int rr = (threadIdx.x >> 5) + j * (NW * 2);
        const bool row_ok = row0 + rr < n_rows;
        const int sample = e_sample[j];
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) v += part[w][rr][cc];
        v += bias;

        if (EPI == EPI_RELU) {
          if (row_ok) ((T*)a.out)[(size_t)sample * a.ldo + col] = Elem<T>::from_f32(fmaxf(v, 0.f));
        } else if (EPI == EPI_LOGITS) {
          if (row_ok && col < a.n_cols) ((float*)a.out)[(size_t)sample * a.ldo + col] = v;
        } else {  // EPI_BERNOULLI: x_t = 1 iff u_t < sigmoid(z_t); count changes per sample
          int cnt = 0;
          if (row_ok && col_live) {
            const float p = 1.0f / (1.0f + expf(-v));
            const uint8_t xn = e_noise[j] < p ? 1 : 0;
            cnt = (xn != e_xold[j]);
            if (cnt) {   // an unchanged symbol (and its encoding) is already in place
              a.x[(size_t)sample * a.D + col] = xn;
              ((T*)a.enc)[(size_t)sample * a.ld_enc + col] = Elem<T>::from_f32((float)xn);
            }
          }
          // the 32 lanes of a half-wave hold one sample row of the tile
          cnt += __shfl_xor(cnt, 1);
          cnt += __shfl_xor(cnt, 2);
          cnt += __shfl_xor(cnt, 4);
          cnt += __shfl_xor(cnt, 8);
          cnt += __shfl_xor(cnt, 16);
          if (cc == 0 && cnt > 0) count_changed(&a.changed[sample], cnt);
        }
      }
    }
  }
  if (EPI == EPI_BERNOULLI && a.retire.enabled) finish_pass(a.retire, gridDim.x);
}

// Gumbel-max draw for categorical positions from logits held in memory:
// x[n, t] = argmax_c (z[n, t, c] + g[n, t, c]), lowest c on ties.  One wave per (row, t).
template <typename T>
__global__ __launch_bounds__(256) void gumbel_argmax_kernel(const float* __restrict__ z, int ldz,
                                                            const float* __restrict__ g, uint8_t* x, T* enc,
                                                            int ld_enc, int* changed, const int* rows,
                                                            const int* n_rows_ptr, int n_rows_fixed, int D, int C,
                                                            int t_lo, int t_hi, RetireArgs retire) {
  const int n_rows = n_rows_ptr ? *n_rows_ptr : n_rows_fixed;
  const int lane = threadIdx.x & 63;
  const int wave_global = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int span = t_hi - t_lo;
  const int row = wave_global / span, t = t_lo + wave_global % span;
  if (row < n_rows) {
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
    if (xn != x[idx]) count_changed(&changed[sample], 1);
    x[idx] = xn;
    enc[(size_t)sample * ld_enc + t] = Elem<T>::from_f32(((float)xn - 128.0f) * (1.0f / 128.0f));
  }
  }
  if (retire.enabled) finish_pass(retire, gridDim.x);
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

__global__ void reset_rows_kernel(int* rows, int* n_rows, int N, int* changed, int* iters, int* flags,
                                  int* done_ctr) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < N) {
    rows[i] = i;
    changed[i] = 0;
    if (iters) iters[i] = 0;
  }
  if (i == 0) {
    *n_rows = N;
    *done_ctr = 0;
    if (flags) *flags = 0;
  }
}

}  // namespace jm
