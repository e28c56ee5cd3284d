// Device code of libjacobi_made.so (gfx950 only).
//
// One Jacobi pass (the loop body of Algorithm 1) is: every hidden masked layer, then the output
// masked layer whose epilogue draws the symbols from the fixed noise (Appendix A.3) and counts,
// per sample, how many positions changed (the forward difference of Section 2.2.1 with
// tolerance 0).  The last workgroup of that kernel retires unchanged samples from the active list.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace jm {

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  Used where an index
// into a register array MUST be a constant (a loop the compiler declines to unroll would push the array,
// e.g. 256 accumulators, into scratch memory).
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

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

// P(x = 1) = 1 / (1 + exp(-v)) of a binary state (the conditional a draw u < P is taken from), evaluated with the
// hardware's exp2 and reciprocal: within 1e-6 of the exact value (|v| log2(e) 2^-24 relative in the exponential,
// scaled by P (1 - P) <= 1/4, plus an ulp each for exp2 and the reciprocal), 0 and 1 at the extremes.  Every
// kernel that draws binary states from logits uses this one expression, so a draw does not depend on which of
// them made it.  (The library's full-precision expf and division cost ~80 instructions per draw.)
__device__ __forceinline__ float bernoulli_probability(float v) { return __builtin_amdgcn_rcpf(1.0f + __expf(-v)); }

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
  static constexpr int EPL = 32;  // elements one lane loads per K chunk (64 bytes)
  static __device__ __forceinline__ bf16_t from_f32(float f) { return f32_to_bf16(f); }
  // 16 bytes = elements v[0..7], ReLU applied (registers only: no array whose address is taken)
  static __device__ __forceinline__ uint4 relu_piece(const float* v) {
    uint4 o;
    o.x = (uint32_t)f32_to_bf16(fmaxf(v[0], 0.f)) | ((uint32_t)f32_to_bf16(fmaxf(v[1], 0.f)) << 16);
    o.y = (uint32_t)f32_to_bf16(fmaxf(v[2], 0.f)) | ((uint32_t)f32_to_bf16(fmaxf(v[3], 0.f)) << 16);
    o.z = (uint32_t)f32_to_bf16(fmaxf(v[4], 0.f)) | ((uint32_t)f32_to_bf16(fmaxf(v[5], 0.f)) << 16);
    o.w = (uint32_t)f32_to_bf16(fmaxf(v[6], 0.f)) | ((uint32_t)f32_to_bf16(fmaxf(v[7], 0.f)) << 16);
    return o;
  }
};
template <> struct Elem<float> {
  static constexpr int EPL = 16;
  static __device__ __forceinline__ float from_f32(float f) { return f; }
  static __device__ __forceinline__ uint4 relu_piece(const float* v) {
    return make_uint4(__float_as_uint(fmaxf(v[0], 0.f)), __float_as_uint(fmaxf(v[1], 0.f)),
                      __float_as_uint(fmaxf(v[2], 0.f)), __float_as_uint(fmaxf(v[3], 0.f)));
  }
};

// Four consecutive elements (dst aligned to them) from four floats: 8 bytes in bf16, 16 in fp32.  bf16 through
// the hardware's conversion (round to nearest even like f32_to_bf16, one instruction per pair instead of six per
// element: at 64 K outputs per workgroup the epilogue of the 256 x 256 kernel is bound by such arithmetic).
template <typename T>
__device__ __forceinline__ void store_quad(T* dst, float a, float b, float c, float d);
template <>
__device__ __forceinline__ void store_quad<bf16_t>(bf16_t* dst, float a, float b, float c, float d) {
  typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  const f32x4_t f = {a, b, c, d};
  *(bf16x4_t*)dst = __builtin_convertvector(f, bf16x4_t);
}
template <>
__device__ __forceinline__ void store_quad<float>(float* dst, float a, float b, float c, float d) {
  *(float4*)dst = make_float4(a, b, c, d);
}

// 16 bytes of a stream that is read once per launch (weights that exceed the caches, noise): loaded with the
// non-temporal hint.  Measured on this chip, a plain read of 2 GiB in contiguous pieces per workgroup: 6.4 TB/s with
// ordinary loads, 7.1 TB/s with these.  Only for loads that take whole 128-byte lines in one instruction: the
// Bernoulli and categorical epilogues fetch a line of noise with four instructions of 16 bytes per lane and lose
// (0.200 against 0.177 ms, 150 against 142 us per launch) when the line is not kept between them.
__device__ __forceinline__ uint4 load_stream16(const uint4* p) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// frag_offset(row, k) = frag_row_offset(row) + frag_col_offset(k): for code that stores many (row, k) pairs
template <typename T>
__device__ __forceinline__ size_t frag_row_offset(int row, int k_chunks) {
  constexpr int KC = 2 * Elem<T>::EPL, P = 16 / (int)sizeof(T);
  return (size_t)(row >> 5) * k_chunks * (size_t)(KC * 32) + (size_t)((row & 31) * P);
}
template <typename T>
__device__ __forceinline__ uint32_t frag_col_offset(int k) {
  constexpr int EPL = Elem<T>::EPL, KC = 2 * EPL, P = 16 / (int)sizeof(T);
  const int c = k / KC, kk = k % KC;
  const int h = kk / EPL, s = (kk % EPL) / P, i = kk % P;
  return (uint32_t)c * (uint32_t)(KC * 32) + (uint32_t)(((s * 2 + h) * 32) * P + i);
}

// Fragment-major layout of every MFMA operand matrix (masked weights, network input, hidden activations).
//
// A [rows, K] matrix is cut into groups of 32 rows and chunks of KC = 2 * EPL columns (128 bytes per row).
// Block (group g, chunk c) holds 32 x KC elements, stored in exactly the order a wave consumes them:
//     [slot s = 0..3][half h = 0..1][row r = 0..31][16 bytes]
// where the 16 bytes are columns  c*KC + h*EPL + s*P .. + P  of row 32*g + r  (P = elements per 16 bytes).
// Lane (r, h) of a wave needs, for MFMA step s, exactly those 16 bytes, so each of the wave's four loads
// per chunk reads one contiguous 1 KB run instead of 64 scattered 16-byte pieces (which makes the
// texture-address path, not memory, the limit).  Blocks are stored chunk-major inside a group.
template <typename T>
__host__ __device__ __forceinline__ size_t frag_offset(int row, int k, int k_chunks) {
  constexpr int EPL = Elem<T>::EPL, KC = 2 * EPL, P = 16 / (int)sizeof(T);
  const int g = row >> 5, r = row & 31, c = k / KC, kk = k % KC;
  const int h = kk / EPL, s = (kk % EPL) / P, i = kk % P;
  return ((size_t)g * k_chunks + c) * (size_t)(KC * 32) + (size_t)(((s * 2 + h) * 32 + r) * P + i);
}

constexpr int TILE = 32;   // output tile: 32 samples x 32 units per workgroup
#ifndef JM_NW
#define JM_NW 8
#endif
#ifndef JM_PD
#define JM_PD 2
#endif
constexpr int NW = JM_NW;  // waves per workgroup; they split the K range between them
constexpr int PD = JM_PD;  // K chunks a wave keeps in flight (all their loads are issued before the first MFMA); <= 8.
                           // 2: ~110 registers, so two workgroups share a compute unit (4 needs ~170: one); equal at
                           // batch 128 (one workgroup per unit anyway), +15-18 % at batches 512-1024
static_assert(PD >= 1 && PD <= 8, "prefetch depth must be 1..8");
constexpr int XCDS = 8;    // workgroup i is dispatched to XCD i % 8; each XCD has its own L2

enum Epilogue { EPI_RELU = 0, EPI_LOGITS = 1, EPI_BERNOULLI = 2, EPI_LOGISTIC = 3 };
// Per-sample changed counters sit one per 128-byte line (index sample * CHG): every workgroup that redraws
// positions of a sample adds to its counter, and atomics on one line are performed one after the other (~1.3 ns
// each), so 128 counters packed into four lines made the ~3000 atomics of a cfg2 pass queue up for a microsecond.
constexpr int CHG = 32;
constexpr float LOGISTIC_A_LO = -6.0f, LOGISTIC_A_HI = 3.0f;   // the log-scale output is clipped to this range

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
  int n_max;             // upper bound of *n_in known to the host (the chain's size): bounds the early read of rows_in
  int* host_flags;       // device-visible pinned host word mirroring *flags (the host reads it after the call's last
                         // kernel has finished)
  int last_pass;
  int flag_unconverged;
  int enabled;
  // Frozen positions (categorical output kernel, see CatArgs::t_first_ptr): fc_in = the word in which this pass's
  // workgroups recorded the lowest position that changed (NULL: not tracked); the tail turns it into the first
  // position the next pass has to evaluate (*t_first_out), tells the host (host_t_first) and re-arms the word the
  // next pass records into (*fc_reset).
  int* fc_in;
  int* t_first_out;
  int* fc_reset;
  int* host_t_first;
};
constexpr int NO_CHANGE = 0x7fffffff;

// Stop test without a tail (short lists, at most DERIVE_MAX_ROWS samples).  retire_tail above costs the pass's last
// kernel three dependent memory round trips after its arithmetic is done (counter atomics performed -> arrival
// counter -> the last workgroup reads the counters).  Instead, the sampling kernel of pass k only ORs one bit per
// changed row into a word per row tile (`LayerArgs::lazy_mask`, by position in pass k's list), and EVERY workgroup
// of the next pass's first kernel derives pass k + 1's list for itself, in LDS, from pass k's list and those words
// -- the same memory round trip in which it would otherwise read the list.  Workgroup 0 also stores the new list and
// count for the pass's other kernels, records the pass counts, clears the mask words of the pass after next and
// reports to the host.  Three sets of mask words rotate: pass k writes set k % 3, pass k + 1 reads it and clears
// set (k + 2) % 3, which was last read a whole pass earlier.
constexpr int DERIVE_MAX_ROWS = 256;
constexpr int DERIVE_WORDS = DERIVE_MAX_ROWS / 32;
static_assert(NW * 64 >= DERIVE_MAX_ROWS + 64, "one thread per list entry, padding included");
struct DeriveArgs {
  int enabled;
  const int* rows_in;       // the previous pass's list and count
  const int* n_in;
  int* rows_out;            // this pass's list and count (written by workgroup 0)
  int* n_out;
  const unsigned* mask_in;  // [DERIVE_WORDS] bit r of word t: row 32 t + r of rows_in changed in the previous pass
  unsigned* mask_clear;     // [DERIVE_WORDS] the set the pass after this one will write
  int* iters;               // per-sample pass counts: the samples of rows_in took pass `pass`
  int pass;
  int n_max;                // upper bound of *n_in known to the host
  int* host_slot;           // pinned host word receiving this pass's active count (= what the previous pass left)
};

struct LayerArgs {
  // operands, both in fragment-major layout with k_chunks chunks per row group:
  // A = activations [sample, K], W = masked weights [unit, K]
  const void* A;
  const void* W;
  int k_chunks;
  const float* bias;     // [out_pad]
  const int* tile_kend;  // per 32-unit tile: K extent that holds non-zero (visible) weights, chunk-rounded
  int k_cap;             // additional upper limit on K (chunk-rounded)
  int k_begin;           // first K element this launch multiplies (chunk-rounded; 32 x 32 tile kernel only).  The
                         // contribution of the inputs before it comes from `partial`:
  const float* partial;  // [sample, ld_partial] fp32 sums over the inputs [0, k_begin) of every unit of the layer, added
  int ld_partial;        // to the tile's own sum before bias and activation; NULL: nothing to add
  int tile_begin;        // first unit tile this launch covers
  int n_launch_tiles;    // unit tiles this launch covers
  int row_tiles;         // sample tiles this launch covers (upper bound; tiles beyond n_rows idle)
  int big_by_rows;       // 256 x 256 kernel only: XCDs own sample tiles (1) or unit tiles (0)
  int io_aligned;        // 256 x 256 kernel only: D % 16 == 0 and noise / x are 16-byte aligned
  // active samples: rows[0 .. *n_rows_ptr) are sample ids (NULL = identity, n_rows fixed)
  const int* rows;
  const int* n_rows_ptr;
  int n_rows;
  int n_rows_pad;        // entries the list `rows` holds (reads past the active count stay inside it)
  // Activations that live only inside one pass can be stored by POSITION in the active list instead of by
  // sample: the layer that reads them then needs no look-up in `rows` before it can request its operands (one
  // dependent memory round trip less per kernel).  a_by_pos: rows of A are list positions; out_by_pos: EPI_RELU
  // writes row (list position) instead of row (sample).
  int a_by_pos, out_by_pos;
  int pos_base;          // first row of this chain's positions (chains run concurrently on disjoint row ranges)
  // EPI_RELU: out = next layer's activations (fragment-major, out_chunks chunks).  EPI_LOGITS: float [sample, ldo]
  void* out;
  int ldo;
  int out_chunks;
  int n_cols;            // real (unpadded) number of units of this layer
  // EPI_BERNOULLI
  const float* noise;    // u[sample, D]
  uint8_t* x;            // [sample, D], updated in place
  void* enc;             // network input of the next pass (fragment-major, enc_chunks chunks)
  int enc_chunks;
  int* changed;          // per-sample count of positions whose symbol changed
  int D;
  int t_lo, t_hi;        // only positions in [t_lo, t_hi) are re-drawn
  // Jacobi-GS (Algorithm 2): the rows are "virtual samples" (block i, sample n) = row i * noise_mod + n, each
  // block carrying its own mixed input.  diag_pos[row tile] is the one position that tile's block draws in
  // this sub-step (-1: none), so the launch evaluates one unit tile per row tile; a virtual sample reads the
  // noise of its real sample.  diag_pos == NULL: an ordinary launch.
  const int* diag_pos;
  int noise_mod, noise_n;
  // EPI_LOGISTIC (continuous states, logistic conditionals): output rows 2t / 2t+1 are the mean and the
  // log-scale of position t; x_t = mean + exp(clip(log-scale)) * l_t with l = noise (standard logistic
  // variates); a position counts as changed when it moved by more than eps.  t_lo / t_hi are positions.
  float* xr;             // [sample, D] real states, updated in place
  float eps;
  RetireArgs retire;
  unsigned* lazy_mask;   // EPI_BERNOULLI: changed rows are recorded as bits here instead of in `changed` (see DeriveArgs)
  DeriveArgs derive;     // EPI_RELU, first layer of a pass: the list comes from the previous pass's mask words
};

// Store that other workgroups of the SAME kernel will read after a grid barrier.  COH = true writes through to
// device-coherent memory (device-scope atomic store: the XCDs' L2 caches are not coherent with each other), so
// that the barrier does not have to write back a whole L2; COH = false is an ordinary store, enough when the
// reader is a later kernel.
template <bool COH, typename V>
__device__ __forceinline__ void publish(V* p, V v) {
  if (COH)
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    *p = v;
}

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

// JM_TSTAMP / JM_STAMP: time-stamp hooks of development builds (-DJM_TRACE); they expand to nothing otherwise.
#include "dev_trace.hpp"

// What the host learns of a pass, written by ONE thread: first the not-converged flag (device copy and its mirror
// in pinned host memory), then the new active count -- the word the host polls.  The host reads the flag mirror as
// soon as it has seen the count of a call's last pass, so the flag must be visible first: the count is stored with
// release semantics in that (rare) case.  Otherwise the host reads nothing but the count before it synchronises
// the stream, and a relaxed store will do.
__device__ __forceinline__ void publish_pass_result(const RetireArgs& r, bool flagged, int new_n) {
  if (flagged) {
    __hip_atomic_fetch_or(r.flags, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (r.host_flags) __hip_atomic_store(r.host_flags, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(r.host_slot, new_n, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  } else {
    __hip_atomic_store(r.host_slot, new_n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

// Stop test and compaction (the forward-difference test of Algorithm 1 with tolerance 0, per
// sample): every active sample took one more pass; those whose symbols changed stay active, in
// order, unless this was the last allowed pass.  Runs in ONE workgroup, after all others finished.
// pre_n / pre_row / pre_iters: *r.n_in, r.rows_in[threadIdx.x] and that sample's pass count, read by every
// workgroup before it reported in (none of them changes during the kernel), so that the one that runs this is
// two dependent memory round trips shorter.
__device__ __forceinline__ void retire_tail(const RetireArgs& r, int pre_n, int pre_row, int pre_iters) {
  __shared__ int wave_total[NW];
  __shared__ int base_s;
  __shared__ int flagged_s;          // some sample was still changing in the last allowed pass
  const int nthreads = blockDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = nthreads >> 6;
  const int n_rows = pre_n;
  if (threadIdx.x == 0) {
    base_s = 0;
    flagged_s = 0;
  }
  __syncthreads();
  if (n_rows <= nthreads) {
    // ---- one row per thread (batches up to a workgroup's size: the latency-critical case)
    const int rix = threadIdx.x;
    int sample = -1;
    bool keep = false;
    if (rix < n_rows) {
      sample = pre_row;
      // counters were built with device-scope atomics by workgroups on other XCDs: read them the same way
      const int c = __hip_atomic_load(&r.changed[(size_t)sample * CHG], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      r.changed[(size_t)sample * CHG] = 0;
      r.iters[sample] = pre_iters + 1;
      keep = (c > 0) && !r.last_pass;
      if (c > 0 && r.last_pass && r.flag_unconverged) flagged_s = 1;   // (every writer stores 1)
    }
    const unsigned long long mask = __ballot(keep);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wave_total[wave] = __popcll(mask);
    __syncthreads();
    int off = 0;
    for (int w = 0; w < wave; ++w) off += wave_total[w];
    if (keep) r.rows_out[off + before] = sample;
    if (threadIdx.x == 0) {
      int tot = 0;
      for (int w = 0; w < nwaves; ++w) tot += wave_total[w];
      base_s = tot;
    }
    __syncthreads();
  } else {
    // ---- large lists: every thread owns a contiguous run of up to 64 rows per round (one round covers
    // 64 * nthreads rows), reads its rows' counters in groups of independent loads, and the kept rows are
    // placed by a prefix sum over the threads' counts: order kept, and the work is spread over the workgroup
    // instead of one dependent round trip per nthreads rows (measured 263 us for 32768 rows that way).
    constexpr int G = 8;
    int base = 0;
    bool unconverged = false;
    for (int s0 = 0; s0 < n_rows; s0 += 64 * nthreads) {
      const int n_here = min(n_rows - s0, 64 * nthreads);
      const int per = (n_here + nthreads - 1) / nthreads;            // <= 64
      const int i0 = min(s0 + n_here, s0 + (int)threadIdx.x * per), i1 = min(s0 + n_here, i0 + per);
      unsigned long long keep = 0;
      for (int g = i0; g < i1; g += G) {
        int sample[G], c[G], itv[G];
#pragma unroll
        for (int q = 0; q < G; ++q) sample[q] = g + q < i1 ? r.rows_in[g + q] : -1;
#pragma unroll
        for (int q = 0; q < G; ++q) {
          c[q] = 0;
          itv[q] = 0;
          if (sample[q] >= 0) {
            c[q] = __hip_atomic_load(&r.changed[(size_t)sample[q] * CHG], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            itv[q] = r.iters[sample[q]];
          }
        }
#pragma unroll
        for (int q = 0; q < G; ++q) {
          if (sample[q] >= 0) {
            r.changed[(size_t)sample[q] * CHG] = 0;
            r.iters[sample[q]] = itv[q] + 1;
            if (c[q] > 0 && !r.last_pass) keep |= 1ull << (g - i0 + q);
            if (c[q] > 0 && r.last_pass && r.flag_unconverged) unconverged = true;
          }
        }
      }
      const int cnt = __popcll(keep);
      int incl = cnt;                                               // inclusive prefix over the wave's lanes
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int v = __shfl_up(incl, d);
        if (lane >= d) incl += v;
      }
      if (lane == 63) wave_total[wave] = incl;
      __syncthreads();
      int off = base + incl - cnt, tot = 0;
      for (int w = 0; w < nwaves; ++w) {
        if (w < wave) off += wave_total[w];
        tot += wave_total[w];
      }
      for (int g = i0; g < i1; g += G) {
        int sample[G];
#pragma unroll
        for (int q = 0; q < G; ++q) sample[q] = (g + q < i1 && ((keep >> (g - i0 + q)) & 1ull)) ? r.rows_in[g + q] : -1;
#pragma unroll
        for (int q = 0; q < G; ++q)
          if (sample[q] >= 0) r.rows_out[off++] = sample[q];
      }
      base += tot;
      __syncthreads();                                              // wave_total is reused by the next round
    }
    if (unconverged) flagged_s = 1;
    if (threadIdx.x == 0) base_s = base;
    __syncthreads();
  }
  // the next pass reads whole tiles of the new list: pad it with a valid id of this call (anything older
  // in those slots may stem from a call with a larger batch)
  if (n_rows > 0) {
    const int fill = r.rows_in[0];
    const int new_n = base_s;
    for (int i = new_n + threadIdx.x; i < ((new_n + 63) & ~63); i += nthreads) r.rows_out[i] = fill;
  }
  if (threadIdx.x == 0) {
    *r.n_out = base_s;
    *r.done_ctr = 0;
    if (r.fc_in) {
      // a sample that goes on changed first at position f >= *fc_in, so its positions up to f read unchanged inputs in
      // the next pass and keep their symbols: the next pass starts behind the lowest f of the batch
      const int fc = __hip_atomic_load(r.fc_in, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int t_first = fc == NO_CHANGE ? NO_CHANGE : fc + 1;
      *r.t_first_out = t_first;
      *r.fc_reset = NO_CHANGE;
      __hip_atomic_store(r.host_t_first, t_first, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    publish_pass_result(r, flagged_s != 0, base_s);
  }
}

// The retire step as a kernel of its own, for lists too long for one workgroup to go through quickly (one
// compute unit handles the scattered counter reads of 32768 rows in ~180 us; spread over the chip they take a
// few us, which repays the extra launch).  Every workgroup takes RETIRE_WG_ROWS consecutive list entries, keeps
// their order, and claims its place in the new list with one atomic add on a cursor: the order of the
// workgroups' runs in the new list is that of their arrival, which no result depends on (every sample's
// arithmetic is independent of its place in the list).  The last workgroup to finish pads and publishes the list.
// cursor = r.done_ctr + RETIRE_CURSOR (a line of its own); both are zero on entry and on exit.
constexpr int RETIRE_WG_ROWS = 1024;
constexpr int RETIRE_CURSOR = 32;
__global__ __launch_bounds__(256) void retire_kernel(RetireArgs r) {
  __shared__ int wave_total[4];
  __shared__ int base_s;
  __shared__ int is_last_s;
  constexpr int Q = RETIRE_WG_ROWS / 256;
  const int n_rows = min(*r.n_in, r.n_max);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int first = blockIdx.x * RETIRE_WG_ROWS + wave * (Q * 64) + lane;   // a wave owns Q * 64 consecutive rows
  int* cursor = r.done_ctr + RETIRE_CURSOR;
  int sample[Q], c[Q], itv[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) sample[q] = first + q * 64 < n_rows ? r.rows_in[first + q * 64] : -1;
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    c[q] = 0;
    itv[q] = 0;
    if (sample[q] >= 0) {
      c[q] = __hip_atomic_load(&r.changed[(size_t)sample[q] * CHG], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      itv[q] = r.iters[sample[q]];
    }
  }
  bool unconverged = false;
  int pos[Q], wave_count = 0;
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    bool keep = false;
    if (sample[q] >= 0) {
      r.changed[(size_t)sample[q] * CHG] = 0;
      r.iters[sample[q]] = itv[q] + 1;
      keep = c[q] > 0 && !r.last_pass;
      unconverged |= c[q] > 0 && r.last_pass && r.flag_unconverged;
    }
    const unsigned long long mask = __ballot(keep);
    pos[q] = keep ? wave_count + __popcll(mask & ((1ull << lane) - 1ull)) : -1;
    wave_count += __popcll(mask);
  }
  if (lane == 0) wave_total[wave] = wave_count;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int tot = wave_total[0] + wave_total[1] + wave_total[2] + wave_total[3];
    base_s = tot ? __hip_atomic_fetch_add(cursor, tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
  }
  __syncthreads();
  int off = base_s;
  for (int w = 0; w < wave; ++w) off += wave_total[w];
#pragma unroll
  for (int q = 0; q < Q; ++q)
    if (pos[q] >= 0) r.rows_out[off + pos[q]] = sample[q];
  // A thread that saw a sample still changing in the last allowed pass sets the device flag and waits for the
  // atomic's result; the barrier then puts every such update of this workgroup before its arrival below, so the
  // workgroup that arrives last finds the flag of all of them.
  if (unconverged) {
    const int old = __hip_atomic_fetch_or(r.flags, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::"v"(old));
  }
  __syncthreads();
  // (thread 0 has its cursor atomic's result, so the atomic below is performed after it; the list entries
  // themselves are read by the next kernel only)
  if (threadIdx.x == 0)
    is_last_s = (__hip_atomic_fetch_add(r.done_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1);
  __syncthreads();
  if (!is_last_s) return;
  const int new_n = __hip_atomic_load(cursor, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (n_rows > 0) {
    // whole tiles of the new list are read by the next pass: pad with a valid id of this call (no other
    // workgroup writes at or behind new_n)
    const int fill = r.rows_in[0];
    for (int i = new_n + threadIdx.x; i < ((new_n + 63) & ~63); i += blockDim.x) r.rows_out[i] = fill;
  }
  if (threadIdx.x == 0) {
    *r.n_out = new_n;
    __hip_atomic_store(cursor, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(r.done_ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int fl = __hip_atomic_load(r.flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    publish_pass_result(r, (fl & 1) != 0 && r.last_pass && r.flag_unconverged, new_n);
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
  const int pre_n = *r.n_in;
  const int pre_row = (int)threadIdx.x < r.n_max ? r.rows_in[threadIdx.x] : 0;
  // (only the retire step writes iters; an empty list reads none: iters may be the caller's memory)
  const int pre_iters = (int)threadIdx.x < min(pre_n, r.n_max) ? r.iters[pre_row] : 0;
  __syncthreads();
  JM_TSTAMP(6, 0);
  if (threadIdx.x == 0)
    is_last_s = (__hip_atomic_fetch_add(r.done_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                 total_workgroups - 1);
  __syncthreads();
  JM_TSTAMP(7, 0);
  if (is_last_s) {
    retire_tail(r, pre_n, pre_row, pre_iters);
    JM_TRACE_TAIL_DONE();
  }
}


// 16 bytes that another workgroup of the SAME kernel may have written (through publish<true>) before the last
// grid barrier: device-scope loads, which are served coherently without this XCD's caches having been
// invalidated as a whole (that would also drop the weights every layer re-reads).
template <bool COH>
__device__ __forceinline__ uint4 load_shared16(const uint4* p) {
  if (!COH) return *p;
  const unsigned long long lo = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long hi = __hip_atomic_load((const unsigned long long*)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
}

// CNT chunks c0, c0 + NW, ... of one wave: every load is issued before the first MFMA.  Ap / Wp point at
// the lane's 16 bytes of slot 0 in chunk 0 of its row group; a chunk is 256 uint4, a slot 64 uint4.
template <typename T, int CNT, bool COH>
__device__ __forceinline__ void chunk_group(const uint4* Ap, const uint4* Wp, int c0, f32x16& acc) {
  static_assert(CNT >= 1 && CNT <= PD, "group larger than the prefetch depth");
  uint4 av[CNT][4], bv[CNT][4];
#pragma unroll
  for (int p = 0; p < CNT; ++p) {
    const uint4* ap = Ap + (size_t)(c0 + p * NW) * 256;
    const uint4* wp = Wp + (size_t)(c0 + p * NW) * 256;
#pragma unroll
    for (int s = 0; s < 4; ++s) { av[p][s] = load_shared16<COH>(ap + s * 64); bv[p][s] = wp[s * 64]; }
  }
  // keep the scheduler from sinking loads between the MFMAs to save registers: the point is to have
  // every load of the group in flight at once
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int p = 0; p < CNT; ++p) mfma_chunk<T>(av[p], bv[p], acc);
}

// One masked dense layer on a 32 x 32 output tile per workgroup.
//
// Lane (r = lane % 32, h = lane / 32) of a wave owns sample row r and weight row r of the tile and
// per K chunk holds 64 bytes of each, the h-th half of the chunk.  The MFMA contracts lane-held K
// slices of A against the same slices of B, so which physical K a slot carries does not matter as
// long as both operands agree.  Both operands live in the fragment-major layout described at
// frag_offset, so every wave-wide load is one contiguous kilobyte.  At batch sizes around 100 a tile's whole K
// range is only a few hundred KB, so the work is bound by memory latency, not by bandwidth or MFMA rate: the waves of a workgroup take K
// chunks round-robin and each issues the loads of up to PD chunks before its first MFMA, which puts
// most of the tile in flight at once.  Partial tiles are summed through LDS in a fixed order
// (deterministic results).
//
// rows/n_rows: the active-sample list (global or LDS memory) and its length; entries past n_rows are
// stale but valid sample ids.  `part` is the workgroup's LDS scratch.  All threads of the workgroup
// call this together; the tile (rel_tile, row0) is uniform.
// XCD_LOCAL: every workgroup that touches this sample's counters runs on the same XCD (see xcd_sampler_kernel), so
// the counter atomics need not leave that XCD's L2: workgroup-scope atomics (atomics are always performed in the
// L2, and all of these workgroups share one) instead of device-scope ones, which go to the memory side.
template <typename T, int EPI, bool COH, bool XCD_LOCAL = false>
__device__ __forceinline__ void compute_tile(const LayerArgs& a, int rel_tile, int row0, const int* rows, int n_rows,
                                             float (*part)[TILE][TILE + 1]) {
  constexpr int EPL = Elem<T>::EPL;
  constexpr int KC = 2 * EPL;
  constexpr int EPT = TILE * TILE / (NW * 64);   // tile elements each thread finishes in the epilogue
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int tile = a.tile_begin + rel_tile;
  const int col0 = tile * TILE;
  const int cc = threadIdx.x & 31, col = col0 + cc;

  JM_TSTAMP(0, 0);
  // Everything that does not depend on other loads is requested up front, so a tile is a chain of only
  // three memory round trips (bookkeeping, operands, results).
  const int my_sample = a.a_by_pos ? a.pos_base + row0 + r : (rows ? rows[row0 + r] : (row0 + r < a.n_rows ? row0 + r : 0));
  int k_end = a.tile_kend[tile];
  const float bias = a.bias[col];
  int e_sample[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int rr = (threadIdx.x >> 5) + j * (NW * 2);
    e_sample[j] = rows ? rows[row0 + rr] : (row0 + rr < a.n_rows ? row0 + rr : 0);
  }
  float e_partial[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j)
    e_partial[j] = a.partial ? a.partial[(size_t)e_sample[j] * a.ld_partial + col] : 0.f;
  // A tile past the active list ends here (uniform).  The count was requested together with the loads above, so
  // looking at it now costs no round trip of its own; and nothing of the caller's memory (noise, symbols) has
  // been touched yet: a pass enqueued speculatively that finds the list empty reads the model's own memory only.
  if (row0 >= n_rows) return;
  float e_noise[EPT];
  uint8_t e_xold[EPT];
  float e_xr[EPT];
  const int pos = EPI == EPI_LOGISTIC ? (col >> 1) : col;     // the position this output column belongs to
  const bool col_live = (EPI == EPI_BERNOULLI || EPI == EPI_LOGISTIC) && pos >= a.t_lo && pos < a.t_hi;
  if (EPI == EPI_LOGISTIC) {
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      e_noise[j] = 0.f;
      e_xr[j] = 0.f;
      if (col_live && (col & 1) == 0) {
        const size_t idx = (size_t)e_sample[j] * a.D + pos;
        e_noise[j] = a.noise[idx];
        e_xr[j] = a.xr[idx];
      }
    }
  }
  if (EPI == EPI_BERNOULLI) {
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      e_noise[j] = 0.f;
      e_xold[j] = 0;
      if (col_live) {
        const size_t idx = (size_t)e_sample[j] * a.D + col;
        const int nrow = a.noise_mod > 0 ? min(e_sample[j] % a.noise_mod, a.noise_n - 1) : e_sample[j];
        e_noise[j] = a.noise[(size_t)nrow * a.D + col];
        if (COH) {   // (see load_shared16) the aligned word that holds the symbol
          const unsigned word = __hip_atomic_load((const unsigned*)((uintptr_t)(a.x + idx) & ~(uintptr_t)3), __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
          e_xold[j] = (uint8_t)(word >> (8 * (unsigned)((uintptr_t)(a.x + idx) & 3)));
        } else {
          e_xold[j] = a.x[idx];
        }
      }
    }
  }

  JM_TSTAMP(1, 1);
  const uint4* Ap = (const uint4*)a.A + (size_t)(my_sample >> 5) * a.k_chunks * 256 + h * 32 + (my_sample & 31);
  const uint4* Wp = (const uint4*)a.W + (size_t)tile * a.k_chunks * 256 + h * 32 + r;
  if (k_end > a.k_cap) k_end = a.k_cap;

  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  // Chunks wave, wave + NW, ... belong to this wave.  They are taken in straight-line groups: all loads of
  // a group are issued before its first MFMA (no branches inside a group, so nothing forces an early wait).
  // (a launch may start behind the inputs whose contribution is cached: see LayerArgs::k_begin)
  const int c_first = a.k_begin / KC;
  const int n_chunks = max((k_end + KC - 1) / KC - c_first, 0);
  const int n_mine = (n_chunks - wave + NW - 1) / NW;   // wave-uniform (scalar)
  int base = 0;
  for (; base + PD <= n_mine; base += PD) chunk_group<T, PD, COH>(Ap, Wp, c_first + base * NW + wave, acc);
  switch (n_mine - base) {
    case 7: chunk_group<T, (PD > 7 ? 7 : 1), COH>(Ap, Wp, c_first + base * NW + wave, acc); break;
    case 6: chunk_group<T, (PD > 6 ? 6 : 1), COH>(Ap, Wp, c_first + base * NW + wave, acc); break;
    case 5: chunk_group<T, (PD > 5 ? 5 : 1), COH>(Ap, Wp, c_first + base * NW + wave, acc); break;
    case 4: chunk_group<T, (PD > 4 ? 4 : 1), COH>(Ap, Wp, c_first + base * NW + wave, acc); break;
    case 3: chunk_group<T, (PD > 3 ? 3 : 1), COH>(Ap, Wp, c_first + base * NW + wave, acc); break;
    case 2: chunk_group<T, (PD > 2 ? 2 : 1), COH>(Ap, Wp, c_first + base * NW + wave, acc); break;
    case 1: chunk_group<T, 1, COH>(Ap, Wp, c_first + base * NW + wave, acc); break;
    default: break;
  }

  JM_TSTAMP(2, 1);
  __shared__ unsigned tile_mask_s;     // rows of this tile with a changed symbol (lazy stop test)
  if (EPI == EPI_BERNOULLI && threadIdx.x == 0) tile_mask_s = 0;
  // acc[i] is the tile element (row = 8*(i/4) + 4*h + i%4, col = r): rows come from A = samples
#pragma unroll
  for (int i = 0; i < 16; ++i) part[wave][(i >> 2) * 8 + h * 4 + (i & 3)][r] = acc[i];
  __syncthreads();
  JM_TSTAMP(3, 1);

  // The changed-count atomics of the EPT rows are issued without waiting for one another; their old values are
  // waited for once, behind the loop (every atomic must have been performed before this workgroup reports in:
  // see finish_pass).  One wait instead of EPT dependent round trips of ~1.2 us each.
  int count_old[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) count_old[j] = 0;
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int rr = (threadIdx.x >> 5) + j * (NW * 2);
    const bool row_ok = row0 + rr < n_rows;
    const int sample = e_sample[j];
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) v += part[w][rr][cc];
    v += e_partial[j];
    v += bias;

    if (EPI == EPI_RELU) {
      if (row_ok)
        publish<COH && !XCD_LOCAL>((T*)a.out + frag_offset<T>(a.out_by_pos ? a.pos_base + row0 + rr : sample, col, a.out_chunks),
                     Elem<T>::from_f32(fmaxf(v, 0.f)));
    } else if (EPI == EPI_LOGITS) {
      if (row_ok && col < a.n_cols) ((float*)a.out)[(size_t)sample * a.ldo + col] = v;
    } else if (EPI == EPI_LOGISTIC) {
      // even lane: mean of position `pos`, odd lane: its log-scale
      const float a_log = __shfl_xor(v, 1);
      int cnt = 0;
      if (row_ok && col_live && (col & 1) == 0) {
        const float xn = v + expf(fminf(fmaxf(a_log, LOGISTIC_A_LO), LOGISTIC_A_HI)) * e_noise[j];
        if (xn != e_xr[j]) {
          publish<COH && !XCD_LOCAL>(a.xr + (size_t)sample * a.D + pos, xn);
          publish<COH && !XCD_LOCAL>((T*)a.enc + frag_offset<T>(sample, pos, a.enc_chunks), Elem<T>::from_f32(xn));
        }
        cnt = !(fabsf(xn - e_xr[j]) <= a.eps);     // (a NaN counts as changed)
      }
      cnt += __shfl_xor(cnt, 1);
      cnt += __shfl_xor(cnt, 2);
      cnt += __shfl_xor(cnt, 4);
      cnt += __shfl_xor(cnt, 8);
      cnt += __shfl_xor(cnt, 16);
      if (cc == 0 && cnt > 0)
        count_old[j] = __hip_atomic_fetch_add(&a.changed[(size_t)sample * CHG], cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {  // EPI_BERNOULLI: x_t = 1 iff u_t < sigmoid(z_t); count changes per sample
      int cnt = 0;
      if (row_ok && col_live) {
        const float p = bernoulli_probability(v);
        const uint8_t xn = e_noise[j] < p ? 1 : 0;
        cnt = (xn != e_xold[j]);
        if (cnt) {   // an unchanged symbol (and its encoding) is already in place
          publish<COH && !XCD_LOCAL>(a.x + (size_t)sample * a.D + col, xn);
          publish<COH && !XCD_LOCAL>((T*)a.enc + frag_offset<T>(sample, col, a.enc_chunks), Elem<T>::from_f32((float)xn));
        }
      }
      // the 32 lanes of a half-wave hold one sample row of the tile
      cnt += __shfl_xor(cnt, 1);
      cnt += __shfl_xor(cnt, 2);
      cnt += __shfl_xor(cnt, 4);
      cnt += __shfl_xor(cnt, 8);
      cnt += __shfl_xor(cnt, 16);
      if (cc == 0 && cnt > 0) {
        if constexpr (XCD_LOCAL)
          count_old[j] = __hip_atomic_fetch_add(&a.changed[(size_t)sample * CHG], cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        else if (a.lazy_mask)
          atomicOr(&tile_mask_s, 1u << rr);
        else
          count_old[j] = __hip_atomic_fetch_add(&a.changed[(size_t)sample * CHG], cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  if (EPI == EPI_BERNOULLI || EPI == EPI_LOGISTIC) {
#pragma unroll
    for (int j = 0; j < EPT; ++j) asm volatile("" ::"v"(count_old[j]));
  }
  if constexpr (EPI == EPI_BERNOULLI && !XCD_LOCAL) {
    if (a.lazy_mask) {   // (uniform) one update per tile; the next kernel reads it, so nobody waits for it here
      __syncthreads();
      if (threadIdx.x == 0 && tile_mask_s)
        __hip_atomic_fetch_or(&a.lazy_mask[row0 / TILE], tile_mask_s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  JM_TSTAMP(4, 0);
  JM_TSTAMP(5, 1);
}

// Map a linear work item to (unit tile, sample tile) so that the sample tiles sharing a weight tile,
// and the unit tiles sharing an activation tile, fall on the same XCD (item i runs on XCD i % 8 when
// items are workgroup indices).  Returns false for padding items.
__device__ __forceinline__ bool item_to_tile(int item, int n_tiles, int row_tiles, int& rel_tile, int& row0) {
  const int xcd = item % XCDS, slot = item / XCDS;
  row0 = (slot % row_tiles) * TILE;
  rel_tile = (slot / row_tiles) * XCDS + xcd;
  return rel_tile < n_tiles;
}

// Stand-alone launch of one layer (one tile per workgroup).  Used when the batch or the model is too
// large for the persistent kernel below, for categorical models and for sequential sampling.
template <typename T, int EPI>
__global__ __launch_bounds__(NW * 64) void masked_layer_kernel(LayerArgs a) {
  __shared__ float part[NW][TILE][TILE + 1];
  int rel_tile, row0;
  if (EPI == EPI_BERNOULLI && a.diag_pos) {   // one unit tile per row tile (see LayerArgs::diag_pos)
    const int j = a.diag_pos[blockIdx.x];
    if (j >= 0) {
      LayerArgs b = a;
      b.t_lo = j;
      b.t_hi = j + 1;
      compute_tile<T, EPI, false>(b, j / TILE - a.tile_begin, blockIdx.x * TILE, a.rows, a.n_rows, part);
    }
  } else if (EPI == EPI_RELU && a.derive.enabled) {
    // this pass's list, derived by every workgroup for itself (see DeriveArgs); NW * 64 >= DERIVE_MAX_ROWS threads
    __shared__ int drv_rows[DERIVE_MAX_ROWS + 64];
    __shared__ int drv_wave[NW];
    const DeriveArgs& d = a.derive;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int n_prev = min(*d.n_in, d.n_max);
    const int sample = t < d.n_max ? d.rows_in[t] : 0;                 // (the list is padded with valid ids)
    const unsigned word = t < DERIVE_MAX_ROWS ? d.mask_in[t >> 5] : 0u;
    const int fill = d.rows_in[0];
    const bool keep = t < n_prev && ((word >> (t & 31)) & 1u);
    const unsigned long long m = __ballot(keep);
    if (lane == 0) drv_wave[wave] = __popcll(m);
    if (t < DERIVE_MAX_ROWS + 64) drv_rows[t] = fill;                  // whole tiles of the list are read
    __syncthreads();
    int off = 0, new_n = 0;
    for (int w = 0; w < NW; ++w) {
      if (w < wave) off += drv_wave[w];
      new_n += drv_wave[w];
    }
    const int pos = off + __popcll(m & ((1ull << lane) - 1ull));
    if (keep) drv_rows[pos] = sample;
    const int padded = (new_n + 63) & ~63;
    if (blockIdx.x == 0) {
      if (keep) d.rows_out[pos] = sample;
      if (t >= new_n && t < padded) d.rows_out[t] = fill;
      if (t < n_prev) d.iters[sample] = d.pass;
      if (t < DERIVE_WORDS) d.mask_clear[t] = 0u;
      if (t == 0) {
        *d.n_out = new_n;
        __hip_atomic_store(d.host_slot, new_n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
    __syncthreads();
    if (item_to_tile(blockIdx.x, a.n_launch_tiles, a.row_tiles, rel_tile, row0))
      compute_tile<T, EPI, false>(a, rel_tile, row0, drv_rows, new_n, part);
  } else if (item_to_tile(blockIdx.x, a.n_launch_tiles, a.row_tiles, rel_tile, row0)) {
    // (the active count is requested here but first looked at inside compute_tile, after the tile's other
    // bookkeeping loads are on their way: one dependent memory round trip less than testing it first)
    const int n_rows = a.n_rows_ptr ? *a.n_rows_ptr : a.n_rows;
    compute_tile<T, EPI, false>(a, rel_tile, row0, a.rows, n_rows, part);
  }
  if ((EPI == EPI_BERNOULLI || EPI == EPI_LOGISTIC) && a.retire.enabled) finish_pass(a.retire, gridDim.x);
}

// ------------------------------------------------------------------------------------------------
// Large-batch variant of the masked layer: 128 x 128 or 256 x 256 (samples x units) per workgroup.
//
// With a thousand and more active samples a layer is a real GEMM and the 32 x 32 tiles above would re-read
// every operand byte from L2 (16 FLOP per byte).  Here 4 waves (2 x 2) each own W x W MFMA tiles (W = 2: 64 x 64
// outputs, 64 accumulator registers; W = 4: 128 x 128, 256 registers); per half K chunk the workgroup copies 2 W
// sample blocks and 2 W weight blocks (2 KB each) into one stage of an LDS ring, and every wave reads its W + W
// fragments per MFMA step from there: 256 resp. 512 FLOP per byte fetched from L2.  Because global memory already
// holds both operands in fragment order, the LDS image is a plain copy and every ds_read_b128 is conflict free.
// W = 2 leaves room for two workgroups per compute unit (64 KB of LDS, ~200 registers), which fill each other's
// barrier, LDS and epilogue waits; it is the faster shape at every batch measured.
// ------------------------------------------------------------------------------------------------
constexpr int BIG_HALF = 128;            // 16-byte pieces of one block in half a chunk (2 of its 4 MFMA steps)

// Workgroup barrier that orders LDS traffic only.  (__syncthreads also waits for every outstanding global load
// of the wave, i.e. it would drain a prefetch ring at every use.)
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// One wave copies 64 x 16 bytes from global memory (one address per lane) straight into LDS at
// lds_byte_address + 16 * lane (wave-uniform address, handed to the instruction in M0).  Written as assembly
// rather than through the compiler's builtin on purpose: the compiler orders every later LDS read behind ALL
// outstanding copies of this kind that it knows of (vmcnt(0)), which serialises a ring of several stages; this
// way it knows of none, and the caller waits (s_waitcnt vmcnt(n), then a barrier) for exactly the stage it reads.
__device__ __forceinline__ void load_to_lds16(const void* src, uint32_t lds_byte_address) {
  uint32_t saved_m0;   // (M0 is the compiler's to use: put it back)
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "v"(src), "s"(lds_byte_address)
               : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

template <typename T>
__device__ __forceinline__ void mfma_step(const uint4& a, const uint4& b, f32x16& acc);
template <>
__device__ __forceinline__ void mfma_step<bf16_t>(const uint4& a, const uint4& b, f32x16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mfma_step<float>(const uint4& a, const uint4& b, f32x16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// W = MFMA tiles per wave and dimension: 4 (256 x 256 per workgroup, one workgroup per compute unit) or 2 (128 x 128:
// a quarter of the LDS and accumulators, two workgroups per compute unit; for batches that would leave most of the
// chip idle on 256-row tiles).
template <typename T, int EPI, int W>
__global__ __launch_bounds__(256, W == 2 ? 2 : 1) void masked_layer_big_kernel(LayerArgs a) {
  constexpr int BIG_W = W, BIG_T = 2 * W, BIG_ROWS = BIG_T * TILE, BIG_STAGE = 2 * BIG_T * BIG_HALF;
  constexpr int KC = 2 * Elem<T>::EPL;
  // ring of four stages, [block 0 .. 2W-1 = samples, 2W .. 4W-1 = units][128] each (one array, run-time stage index)
  __shared__ uint4 big_ring[4 * BIG_STAGE];
  const int n_rows = a.n_rows_ptr ? *a.n_rows_ptr : a.n_rows;
  const int big_cols = (a.n_launch_tiles + BIG_T - 1) / BIG_T;
  // The visible K grows about linearly with the unit index (units are laid out by degree, positions in order): the
  // last column of unit tiles costs several times the first.  A workgroup therefore takes TWO columns of its sample
  // tile, c from the end and c from the start, one after the other: every workgroup then has about the same work
  // (with one column each and four workgroups per compute unit the slowest unit took 1.45x the average).
  const int pair_cols = (big_cols + 1) / 2;
  // Workgroup i runs on XCD i % 8.  An XCD should own whichever operand is larger (it then streams only
  // the smaller one through its L2): sample tiles when samples outnumber units, unit tiles otherwise.
  const int xcd = blockIdx.x % XCDS, slot = blockIdx.x / XCDS;
  int wg_m, wg_p;                                           // row_tiles counts 256-sample tiles here
  if (a.big_by_rows) {
    wg_p = slot % pair_cols;
    wg_m = (slot / pair_cols) * XCDS + xcd;
  } else {
    wg_m = slot % a.row_tiles;
    wg_p = (slot / a.row_tiles) * XCDS + xcd;
  }
  const int row0 = wg_m * BIG_ROWS;
  if (wg_p < pair_cols && wg_m < a.row_tiles && row0 < n_rows) {
   for (int part = 0; part < 2; ++part) {
    const int wg_n = part == 0 ? big_cols - 1 - wg_p : wg_p;
    if (part == 1 && wg_n >= big_cols - 1 - wg_p) break;     // (an odd number of columns: the middle one is part 0's)
    // (the thread index is made opaque per part: otherwise everything the epilogue derives from it alone is computed
    // once, ahead of the first part, and kept in registers through both main loops, which then spill)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1, wave_in_sub = wave & 1;
    const int rel_tile0 = wg_n * BIG_T;
    const int tile0 = a.tile_begin + rel_tile0;
    const int live_tiles = min(BIG_T, a.n_launch_tiles - rel_tile0);

    int k_end = 0;
    for (int j = 0; j < live_tiles; ++j) k_end = max(k_end, a.tile_kend[tile0 + j]);
    if (k_end > a.k_cap) k_end = a.k_cap;
    const int n_chunks = (k_end + KC - 1) / KC;
    const size_t group = (size_t)a.k_chunks * 256;

    // Operand blocks go from global memory straight into LDS (global_load_lds_dwordx4: lane i of a wave
    // deposits its 16 bytes at the wave's LDS base + 16 i), so data in flight costs no registers.  A chunk is
    // moved in two halves (MFMA steps 0-1 and 2-3 of all 4 W blocks: 32 KB at W = 4) through a ring of four stages,
    // three halves in flight while one is multiplied: a load has three halves' worth of MFMA time (~1.3 us) to
    // arrive.  The copies are issued as assembly (see load_to_lds16), so the compiler knows of none of them: written
    // with the builtin, it ordered every LDS read behind all outstanding LDS-bound loads (a full vmcnt(0) in front
    // of each half's first read, right behind the prefetch it had just issued: load and multiply never overlapped,
    // 2.4 us per chunk instead of < 1).  The waits are written by hand below.  Each thread copies 2 W pieces of
    // 16 bytes per half: element e = half * 128 + (tid & 127) of blocks 2 q + (tid >> 7); offsets in 16-byte units
    // (the host refuses operand buffers of 64 GiB and more).
    // (Requesting the second column's first halves ahead of the first column's epilogue gains nothing: the
    // epilogue's own loads then queue behind 128 KB of copies, and the copies' addresses, kept across the epilogue,
    // are spilled and reloaded with compiler-placed waits that drain the ring inside the main loop.)
    const int sub = wave >> 1, e_lo = tid & 127;             // (sub: wave-uniform)
    uint32_t offA[BIG_W];
#pragma unroll
    for (int q = 0; q < BIG_W; ++q) {
      const int row = row0 + (2 * q + sub) * TILE + (tid & 31);
      const int sample = a.rows ? a.rows[min(row, a.n_rows_pad - 1)] : (row < a.n_rows ? row : 0);
      offA[q] = (uint32_t)((size_t)(sample >> 5) * group) + (e_lo & ~31) + (sample & 31);
    }
    const uint4* Abase = (const uint4*)a.A;
    const uint4* Wbase = (const uint4*)a.W + (size_t)tile0 * group + e_lo;
    const int last_live = live_tiles - 1;                     // tiles past the layer's end repeat the last one
    const int n_half = 2 * n_chunks;

    f32x16 acc[BIG_W][BIG_W];
#pragma unroll
    for (int i = 0; i < BIG_W; ++i)
#pragma unroll
      for (int j = 0; j < BIG_W; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // half hc (clamped to the last one: the ring is always kept full, so that the number of loads in flight is
    // the same at every wait; the surplus copies land in stages nobody reads any more) -> stage array dst
    auto issue_half = [&](int hc, uint4* dst) {
      hc = min(hc, n_half - 1);
      const uint32_t co = (uint32_t)(hc >> 1) * 256 + (uint32_t)(hc & 1) * 128;
      const uint32_t d = lds_address(dst + sub * BIG_HALF + wave_in_sub * 64);
#pragma unroll
      for (int q = 0; q < BIG_W; ++q) {
        load_to_lds16(Abase + offA[q] + co, d + 2 * q * BIG_HALF * 16);
        load_to_lds16(Wbase + (size_t)min(2 * q + sub, last_live) * group + co, d + (BIG_T + 2 * q) * BIG_HALF * 16);
      }
    };
    // A half is multiplied in two sub-steps (MFMA step sl = 0, 1 of its blocks).  The fragments of a sub-step are
    // read from LDS one sub-step ahead, into the register set the sub-step before last has finished with, so the
    // matrix cores always have a sub-step's worth of MFMAs (2 W^2 of them) whose operands are already in registers
    // while the next reads are under way -- with one wave per SIMD nothing else would cover the LDS latency:
    //   read set 1 <- half h, sl 1 | MFMAs on set 0 (half h, sl 0) | barrier, refill, read set 0 <- half h + 1, sl 0 |
    //   MFMAs on set 1
    JM_WAIT_DECL();
    uint4 fa0[BIG_W], fb0[BIG_W], fa1[BIG_W], fb1[BIG_W];
    auto read_frags = [&](const uint4* cur, int sl, uint4 (&fa)[BIG_W], uint4 (&fb)[BIG_W]) {
#pragma unroll
      for (int i = 0; i < BIG_W; ++i) fa[i] = cur[(wm * BIG_W + i) * BIG_HALF + sl * 64 + lane];
#pragma unroll
      for (int j = 0; j < BIG_W; ++j) fb[j] = cur[(BIG_T + wn * BIG_W + j) * BIG_HALF + sl * 64 + lane];
    };
    auto multiply = [&](const uint4 (&fa)[BIG_W], const uint4 (&fb)[BIG_W]) {
#pragma unroll
      for (int i = 0; i < BIG_W; ++i)
#pragma unroll
        for (int j = 0; j < BIG_W; ++j) mfma_step<T>(fb[j], fa[i], acc[i][j]);   // (units = rows of the result)
    };
    // One half.  On entry its sl-0 fragments are on their way into set 0.  The barrier in the middle says: this
    // wave's copies of half hc + 1 have landed (the 2 x 2 W younger ones may still fly), everybody's have, and
    // everybody has read all it needs of half hc (lgkmcnt(0): both of its fragment sets have arrived), so half
    // hc + 4 can be requested into its stage.
    // (no fence there on purpose: a release fence on LDS makes the compiler wait for ALL LDS-bound loads, the
    // younger halves included.  The memory clobber keeps the compiler from moving LDS reads across.)
    auto half_step = [&](int hc, uint4* cur, const uint4* next) {
      read_frags(cur, 1, fa1, fb1);
      __builtin_amdgcn_sched_barrier(0);
      multiply(fa0, fb0);
      __builtin_amdgcn_sched_barrier(0);
      JM_WAIT_BEGIN();
      if constexpr (W == 4) asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
      JM_WAIT_END();
      issue_half(hc + 4, cur);
      read_frags(next, 0, fa0, fb0);
      __builtin_amdgcn_sched_barrier(0);
      multiply(fa1, fb1);
      __builtin_amdgcn_sched_barrier(0);
    };
    JM_TSTAMP(EPI == EPI_RELU ? 0 : 3, 0);
    if (n_half > 0) {
      for (int hc = 0; hc < 4; ++hc) issue_half(hc, big_ring + hc * BIG_STAGE);
      if constexpr (W == 4) asm volatile("s_waitcnt vmcnt(24)\n\ts_barrier" ::: "memory");   // half 0 is there
      else asm volatile("s_waitcnt vmcnt(12)\n\ts_barrier" ::: "memory");
      read_frags(big_ring, 0, fa0, fb0);
      for (int hc = 0; hc < n_half; ++hc)
        half_step(hc, big_ring + (hc & 3) * BIG_STAGE, big_ring + ((hc + 1) & 3) * BIG_STAGE);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // surplus copies: the epilogue reuses stage 0
    __syncthreads();
    // New names for the accumulators from here on: the (long, fully unrolled) epilogue's register needs then do
    // not reach back into the main loop (without this the compiler moved accumulators between register files
    // and reloaded spilled ones inside the loop of the sampling variant).
#pragma unroll
    for (int i = 0; i < BIG_W; ++i)
#pragma unroll
      for (int j = 0; j < BIG_W; ++j) asm volatile("" : "+a"(acc[i][j]));

    JM_TSTAMP(EPI == EPI_RELU ? 1 : 4, 0);
    JM_TRACE_VALUE(EPI == EPI_RELU ? 6 : 7, JM_WAIT_PACK(n_chunks));
    // ---- epilogue.  Four units of a sample are contiguous in every array it touches (noise, symbols, and the
    // fragment-major activations: half of a 16-byte piece in bf16, a whole one in fp32), so results leave the
    // registers in 8- and 16-byte pieces without a transposition through LDS.  The operand stages are free now: the
    // workgroup's 256 sample ids go through stage 0.
    int* ids = (int*)big_ring;
    {
      const int row = row0 + tid;
      if (tid < BIG_ROWS) ids[tid] = row < n_rows ? (a.rows ? a.rows[row] : row) : -1;
    }
    __syncthreads();
    // The weights were the MFMA's row operand, so lane (r, h) holds ONE sample per sample tile and runs of four
    // consecutive units: acc[i][j][e] belongs to sample row0 + (wm*4 + i)*32 + r and unit
    // (tile0 + wn*4 + j)*32 + 8*(e/4) + 4*h + e%4.  Everything the epilogue reads is requested before anything is
    // stored where possible (the bias: here, once for all sample tiles).
    int col_of[BIG_W];                                 // first unit of this lane in unit tile j (+ 8 g per run of four)
    bool tile_ok[BIG_W];
    float4 b4[BIG_W][4];
    uint32_t frag_col[BIG_W][4];                       // the runs' places inside a row of the fragment-major output
#pragma unroll
    for (int j = 0; j < BIG_W; ++j) {
      const int rel_tile = rel_tile0 + wn * BIG_W + j;
      col_of[j] = (a.tile_begin + min(rel_tile, a.n_launch_tiles - 1)) * TILE + 4 * h;
      tile_ok[j] = rel_tile < a.n_launch_tiles;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        b4[j][g] = *(const float4*)(a.bias + col_of[j] + 8 * g);
        frag_col[j][g] = frag_col_offset<T>(col_of[j] + 8 * g);
      }
    }
    if constexpr (EPI == EPI_BERNOULLI) {
      // Sampling, in 8 batches of two unit tiles (8 runs of four positions per lane).  A run that lies wholly inside
      // the window and the row takes the fast path: one 16-byte read of noise, one word of symbols in, one out, one
      // piece of the encoded input (instead of a byte and an element per changed position: the first pass from
      // zeros changes every other one, 26 M single stores at batch 32768).  The inputs of batch b + 1 are requested
      // before the results of batch b are stored: the compiler keeps a load behind every earlier store it cannot
      // prove to be to other memory, and a batch's loads waited for on their own cost a memory round trip each.
      const bool vec_io = a.io_aligned != 0;           // 16-byte reads of noise, 4-byte symbol words: aligned rows
      constexpr int PAIRS = BIG_W / 2, NB = BIG_W * PAIRS;   // unit-tile pairs per sample tile; batches
      bool fast[2][8];
      float4 u4[2][8];
      uint32_t xo[2][8];
      int old_count[BIG_W];                            // what the counter atomics returned: waited for once, at the end
      auto request = [&](int b, bool (&f)[8], float4 (&u)[8], uint32_t (&x)[8]) {
        const int sample = ids[(wm * BIG_W + b / PAIRS) * TILE + r];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int j = 2 * (b % PAIRS) + (q >> 2), col0 = col_of[j] + 8 * (q & 3);
          f[q] = tile_ok[j] && sample >= 0 && vec_io && col0 >= a.t_lo && col0 + 4 <= min(a.t_hi, a.D);
          // (unconditional loads from an address that is always valid: a load inside a branch is waited for there)
          const size_t idx = f[q] ? (size_t)sample * a.D + col0 : 0;
          u[q] = *(const float4*)(a.noise + idx);
          x[q] = *(const uint32_t*)(a.x + idx);
        }
      };
      request(0, fast[0], u4[0], xo[0]);
      int cnt = 0;
      static_for<NB>([&](auto Bt) {
        constexpr int b = decltype(Bt)::value, i = b / PAIRS, pair = b % PAIRS;
        const int sample = ids[(wm * BIG_W + i) * TILE + r];
        const size_t frag_row = frag_row_offset<T>(max(sample, 0), a.enc_chunks);
        if (b + 1 < NB) request(b + 1, fast[(b + 1) & 1], u4[(b + 1) & 1], xo[(b + 1) & 1]);
        if (pair == 0) cnt = 0;
        static_for<8>([&](auto Qt) {
          constexpr int q = decltype(Qt)::value, j = 2 * pair + (q >> 2), g = q & 3;
          const int col0 = col_of[j] + 8 * g;
          const float v[4] = {acc[i][j][4 * g + 0] + b4[j][g].x, acc[i][j][4 * g + 1] + b4[j][g].y,
                              acc[i][j][4 * g + 2] + b4[j][g].z, acc[i][j][4 * g + 3] + b4[j][g].w};
          if (fast[b & 1][q]) {
            const size_t idx = (size_t)sample * a.D + col0;
            const float u[4] = {u4[b & 1][q].x, u4[b & 1][q].y, u4[b & 1][q].z, u4[b & 1][q].w};
            uint32_t xn = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) xn |= (u[c] < bernoulli_probability(v[c]) ? 1u : 0u) << (8 * c);
            if (xn != xo[b & 1][q]) {
              uint32_t d = xn ^ xo[b & 1][q];                      // differing positions: one bit per non-zero byte
              d |= d >> 4;
              d |= d >> 2;
              d |= d >> 1;
              cnt += __popc(d & 0x01010101u);
              *(uint32_t*)(a.x + idx) = xn;
              store_quad<T>((T*)a.enc + (frag_row + frag_col[j][g]), (float)(xn & 1u), (float)((xn >> 8) & 1u),
                            (float)((xn >> 16) & 1u), (float)(xn >> 24));
            }
          } else if (tile_ok[j] && sample >= 0 && col0 < a.t_hi && col0 + 4 > a.t_lo && col0 < a.D) {
            const size_t idx = (size_t)sample * a.D + col0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const int col = col0 + c;
              if (col >= a.t_lo && col < a.t_hi && col < a.D) {
                const uint8_t xn = a.noise[idx + c] < bernoulli_probability(v[c]) ? 1 : 0;
                if (xn != a.x[idx + c]) {
                  cnt++;
                  a.x[idx + c] = xn;
                  ((T*)a.enc)[frag_offset<T>(sample, col, a.enc_chunks)] = Elem<T>::from_f32((float)xn);
                }
              }
            }
          }
        });
        if (pair == PAIRS - 1) {   // the sample tile is done: one counter update by the first of the sample's two lanes
          cnt += __shfl_xor(cnt, 32);
          old_count[i] = 0;
          if (h == 0 && cnt > 0 && sample >= 0)
            old_count[i] = __hip_atomic_fetch_add(&a.changed[(size_t)sample * CHG], cnt, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
        }
      });
      // (the atomics have been performed once their old values are here: see count_changed)
#pragma unroll
      for (int i = 0; i < BIG_W; ++i) asm volatile("" ::"v"(old_count[i]));
    } else {
      static_for<BIG_W>([&](auto I) {
        constexpr int i = decltype(I)::value;
        const int sample = ids[(wm * BIG_W + i) * TILE + r];
        const size_t frag_row = frag_row_offset<T>(max(sample, 0), a.out_chunks);
        static_for<BIG_W>([&](auto J) {
          constexpr int j = decltype(J)::value;
          const bool ok = tile_ok[j] && sample >= 0;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int col0 = col_of[j] + 8 * g;                    // this lane's units col0 .. col0 + 3
            const float v[4] = {acc[i][j][4 * g + 0] + b4[j][g].x, acc[i][j][4 * g + 1] + b4[j][g].y,
                                acc[i][j][4 * g + 2] + b4[j][g].z, acc[i][j][4 * g + 3] + b4[j][g].w};
            if (EPI == EPI_RELU) {
              if (ok) store_quad<T>((T*)a.out + (frag_row + frag_col[j][g]), fmaxf(v[0], 0.f), fmaxf(v[1], 0.f),
                                    fmaxf(v[2], 0.f), fmaxf(v[3], 0.f));
            } else {
              if (ok) {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                  if (col0 + c < a.n_cols) ((float*)a.out)[(size_t)sample * a.ldo + col0 + c] = v[c];
              }
            }
          }
        });
      });
    }
    JM_TSTAMP(EPI == EPI_RELU ? 2 : 5, 1);
    __syncthreads();                                           // (the sample ids in stage 0 make way for operands)
   }
  }
  if (EPI == EPI_BERNOULLI && a.retire.enabled) finish_pass(a.retire, gridDim.x);
}

// ------------------------------------------------------------------------------------------------
// Persistent kernel: the whole of Algorithm 1 (or Algorithm 3) in one cooperative launch.
//
// At batch ~100 a pass is three layers of a few microseconds each, and a dependent kernel launch
// costs about as much as a layer.  Here one workgroup per CU stays resident for the entire call;
// layers are separated by a grid-wide barrier instead of a kernel boundary, the stop test and the
// compaction of the active list are recomputed by every workgroup from the per-sample changed
// counters (identical inputs, identical result, no extra barrier), and the host synchronises once.
// ------------------------------------------------------------------------------------------------
constexpr int PERSIST_MAX_N = 2048;       // active list is kept in LDS
constexpr int PERSIST_MAX_LAYERS = 8;

struct PersistLayer {
  const void* W;
  const float* bias;
  const int* tile_kend;
  const int* cnt_lt;     // hidden layers: cnt_lt[t] = units of degree < t (prefix length); NULL for the output layer
  void* out;             // hidden layers: activation buffer [sample, ldo]
  int in_pad, k_chunks, out_chunks, n_tiles, out_dim;
};

struct PersistArgs {
  PersistLayer layer[PERSIST_MAX_LAYERS];
  int L;                 // hidden layers; layer[L] is the output layer
  void* enc;
  int enc_chunks;
  const float* noise;
  const uint8_t* x_init;
  uint8_t* x;
  int N, D;
  int block;             // GS-Jacobi block size; >= D means plain Jacobi (one block)
  int cap;               // plain Jacobi: pass limit (<= D)
  int flag_unconverged;
  int* changed;          // [2][n_pad] per-sample changed counters, alternating by pass
  int n_pad;
  int* iters;            // [N]
  int* flags;            // bit 0 unconverged, bit 1 barrier timed out
  unsigned* bar;         // grid barrier arrival counter (zero at launch)
  long long* stats;      // [0] passes, [1] sample-passes
  unsigned spin_limit;   // barrier gives up after this many polls (never reached unless the launch was not co-resident)
  // xcd_sampler_kernel: nothing is reset between calls.  Barrier numbers continue where the XCD's previous call
  // left them (a word behind the flag and registration arrays), registration counts continue from reg_base = calls
  // so far x workgroups per XCD, and each XCD reports into its own 8 words of pinned host memory: [0..1] passes,
  // [2..3] sample-passes (64 bit each), [4] flags, [5] = call_id once the rest is written; word 64 collects the
  // back-out flags (2, 4) of all XCDs.
  unsigned reg_base;
  int call_id;
  int* host_report;
};

// Grid-wide barrier for a cooperative (co-resident) launch.  Everything a workgroup wrote for others went
// out through publish<true> (write-through, device scope); each thread waits until its stores are
// acknowledged, then thread 0 arrives and polls until all workgroups have arrived.  Readers use device-scope
// loads (load_shared16 and the like) for whatever another workgroup may have written, so no cache is written
// back or invalidated here.  (A device-scope release fence instead would write back the whole L2 once per
// arriving workgroup, 32 times per XCD and barrier, stalling the workgroups still at work; an acquire fence
// would drop the weights the next layer re-reads.)
// The wait is bounded: on timeout bit 1 of *flags is set and every workgroup leaves the kernel at its next
// check, so the grid always drains.
#ifndef JM_SLEEP
#define JM_SLEEP 1
#endif

__device__ __forceinline__ bool grid_barrier(unsigned* bar, unsigned& epoch, int* flags, unsigned spin_limit) {
  __shared__ int ok_s;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    epoch += gridDim.x;
    JM_STAMP(1);
    JM_STAMP(2);
    __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    JM_STAMP(3);
    int ok = 1;
    unsigned spins = 0;
    while ((int)(__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) < 0) {
      __builtin_amdgcn_s_sleep(JM_SLEEP);
      if (++spins > spin_limit ||
          ((spins & 255) == 0 && (__hip_atomic_load(flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 2))) {
        __hip_atomic_fetch_or(flags, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = 0;
        break;
      }
    }
    JM_STAMP(4);
#ifdef JM_BARRIER_ACQUIRE   // (not needed: everything read across the barrier is read with device-scope loads)
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
#endif
    JM_STAMP(5);
    ok_s = ok;
  }
  __syncthreads();
  return ok_s != 0;
}

template <typename T>
__global__ __launch_bounds__(NW * 64) void persistent_sampler_kernel(PersistArgs p) {
  __shared__ float part[NW][TILE][TILE + 1];
  __shared__ int rows_s[PERSIST_MAX_N];
  __shared__ int wave_total[NW];
  constexpr int NT = NW * 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned epoch = 0;
  const int N = p.N, D = p.D, L = p.L;

  // x = x_init (or zeros) and its network encoding
  for (size_t i = (size_t)blockIdx.x * NT + threadIdx.x; i < (size_t)N * D; i += (size_t)gridDim.x * NT) {
    const int n = (int)(i / D), t = (int)(i % D);
    const uint8_t v = p.x_init ? p.x_init[i] : 0;
    publish<true>(p.x + i, v);
    publish<true>((T*)p.enc + frag_offset<T>(n, t, p.enc_chunks), Elem<T>::from_f32((float)v));
  }
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < N; i += NT) p.iters[i] = 0;
    for (int i = threadIdx.x; i < 2 * p.n_pad; i += NT) publish<true>(p.changed + (size_t)i * CHG, 0);
  }
  if (!grid_barrier(p.bar, epoch, p.flags, p.spin_limit)) return;

  long long n_passes = 0, n_sample_passes = 0;
  int parity = 0;
  const bool gs = p.block < D;
  for (int a0 = 0; a0 < D; a0 += p.block) {
    const int b0 = min(a0 + p.block, D);          // block = 0-based positions [a0, b0)
    // entries past the active count are read as sample ids too (their results are discarded), so the whole
    // padded list must hold valid ids
    for (int i = threadIdx.x; i < PERSIST_MAX_N; i += NT) rows_s[i] = i < N ? i : 0;
    int n_rows = N;
    __syncthreads();
    const int cap = gs ? (b0 - a0) : p.cap;
    for (int k = 1; k <= cap && n_rows > 0; ++k) {
      const int row_tiles = (n_rows + TILE - 1) / TILE;
      int* changed = p.changed + (size_t)parity * p.n_pad * CHG;
      // ---- hidden layers (GS: only units of degree < b0 matter to positions <= b0)
      int in_limit = gs ? b0 - 1 : -1;
      for (int l = 0; l < L; ++l) {
        const PersistLayer& ly = p.layer[l];
        LayerArgs a = {};
        a.A = l == 0 ? p.enc : p.layer[l - 1].out;
        a.W = ly.W;
        a.k_chunks = ly.k_chunks;
        a.bias = ly.bias;
        a.tile_kend = ly.tile_kend;
        a.k_cap = ly.in_pad;
        if (in_limit >= 0) a.k_cap = min(ly.in_pad, (in_limit + 2 * Elem<T>::EPL - 1) / (2 * Elem<T>::EPL) * (2 * Elem<T>::EPL));
        a.tile_begin = 0;
        a.n_rows = N;
        a.out = ly.out;
        a.out_chunks = ly.out_chunks;
        a.n_cols = ly.out_dim;
        int tiles = ly.n_tiles;
        if (gs) {
          const int lim = ly.cnt_lt[b0];
          tiles = min(tiles, (lim + TILE - 1) / TILE);
          in_limit = lim;
        }
        const int groups = (tiles + XCDS - 1) / XCDS;
        const int items = groups * XCDS * row_tiles;
        for (int item = blockIdx.x; item < items; item += gridDim.x) {
          int rel_tile, row0;
          if (item_to_tile(item, tiles, row_tiles, rel_tile, row0)) {
            compute_tile<T, EPI_RELU, true>(a, rel_tile, row0, rows_s, n_rows, part);
            __syncthreads();   // `part` is reused by the next item
          }
        }
        if (!grid_barrier(p.bar, epoch, p.flags, p.spin_limit)) return;
      }
      // ---- output layer with the sampling epilogue, positions [a0, b0)
      {
        const PersistLayer& ly = p.layer[L];
        LayerArgs a = {};
        a.A = p.layer[L - 1].out;
        a.W = ly.W;
        a.k_chunks = ly.k_chunks;
        a.bias = ly.bias;
        a.tile_kend = ly.tile_kend;
        a.k_cap = ly.in_pad;
        if (in_limit >= 0) a.k_cap = min(ly.in_pad, (in_limit + 2 * Elem<T>::EPL - 1) / (2 * Elem<T>::EPL) * (2 * Elem<T>::EPL));
        a.tile_begin = a0 / TILE;
        a.n_rows = N;
        a.n_cols = ly.out_dim;
        a.noise = p.noise;
        a.x = p.x;
        a.enc = p.enc;
        a.enc_chunks = p.enc_chunks;
        a.changed = changed;
        a.D = D;
        a.t_lo = a0;
        a.t_hi = b0;
        const int tiles = (b0 + TILE - 1) / TILE - a.tile_begin;
        const int groups = (tiles + XCDS - 1) / XCDS;
        const int items = groups * XCDS * row_tiles;
        for (int item = blockIdx.x; item < items; item += gridDim.x) {
          int rel_tile, row0;
          if (item_to_tile(item, tiles, row_tiles, rel_tile, row0)) {
            compute_tile<T, EPI_BERNOULLI, true>(a, rel_tile, row0, rows_s, n_rows, part);
            __syncthreads();
          }
        }
        if (!grid_barrier(p.bar, epoch, p.flags, p.spin_limit)) return;
      }
      // ---- stop test and compaction, recomputed identically by every workgroup.  Workgroup 0 also keeps
      //      the per-sample pass counts and clears the counters the pass after next will use (every
      //      workgroup finished reading those before it arrived at this pass's barriers).
      n_passes += 1;
      n_sample_passes += n_rows;
      const bool last_pass = (k == cap);
      int new_n = 0;
      for (int start = 0; start < n_rows; start += NT) {
        const int rix = start + threadIdx.x;
        int sample = -1;
        bool keep = false;
        if (rix < n_rows) {
          sample = rows_s[rix];
          const int c = __hip_atomic_load(&changed[(size_t)sample * CHG], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          keep = (c > 0) && !last_pass;
          if (blockIdx.x == 0) {
            p.iters[sample] += 1;
            if (c > 0 && last_pass && p.flag_unconverged) atomicOr(p.flags, 1);
          }
        }
        const unsigned long long mask = __ballot(keep);
        const int before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_total[wave] = __popcll(mask);
        __syncthreads();                       // all reads of this chunk of rows_s are done
        int off = new_n;
        for (int w = 0; w < wave; ++w) off += wave_total[w];
        if (keep) rows_s[off + before] = sample;   // off + before <= rix: never overtakes an unread entry
        for (int w = 0; w < NW; ++w) new_n += wave_total[w];
        __syncthreads();
      }
      if (blockIdx.x == 0) {
        int* other = p.changed + (size_t)(parity ^ 1) * p.n_pad * CHG;
        for (int i = threadIdx.x; i < N; i += NT) publish<true>(other + (size_t)i * CHG, 0);
      }
      n_rows = new_n;
      parity ^= 1;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    p.stats[0] = n_passes;
    p.stats[1] = n_sample_passes;
  }
}

// ------------------------------------------------------------------------------------------------
// Whole call in one launch, XCD by XCD.
//
// Samples are independent systems, so nothing forces the workgroups of a whole-call kernel to synchronise across
// the chip: XCD g (its 32 compute units share one L2) takes the samples [g * per, (g + 1) * per) through every
// pass of Algorithm 1 / every block of Algorithm 3 on its own.  What its workgroups exchange -- activations,
// symbols, changed counters -- is written by ordinary stores (the vector L1 writes through to the L2) and made
// visible by waiting for those stores and a barrier among the XCD's workgroups on flag words that only they touch;
// readers fetch it with device-scope loads, which go past their unit's L1 and are served by the L2 the writers
// share with them.  (Two cheaper-looking ways to keep stale L1 lines out were tried: invalidating the L1 at every
// barrier with workgroup scope does nothing on this chip outside threadgroup-split mode -- results went wrong --
// and with device scope it made a phase cost 20 us.)  Nothing crosses to another XCD's L2, which is what made
// each phase of the device-wide persistent kernel cost 10-15 us; here a phase is ~7 us on the D = 784, 2 x 2000
// network (against 4.5-8 us for a launch of the per-layer kernels) and ~4 us on small ones.  A workgroup learns
// its XCD from the hardware's XCC id; the scheme needs gridDim / 8 workgroups on each of the 8 XCDs, all
// resident at once.  If that does not hold the whole grid
// backs out (flag 4: surplus workgroup on an XCD; flag 2: a barrier's bounded wait ran out), so the grid always
// drains, and the host takes the per-layer path instead.
// ------------------------------------------------------------------------------------------------
constexpr int XCD_MAX_ROWS = 256;        // samples one XCD takes (its active list is kept in LDS)
constexpr int XCD_LINE = 64;             // words per XCD in the barrier's flag array (one per workgroup of the XCD) and in the
                                         // registration array: two cache lines that only this XCD's workgroups touch

// Barrier among the n_group workgroups of one XCD.  Every workgroup owns one word of the XCD's flag array and
// stores the number of the barrier it has reached there (after its threads' earlier stores have reached the L2);
// the first wave of every workgroup then reads all the words with ONE load per poll (device-scope loads, served
// by the L2 past this unit's L1) until none is behind.  No read-modify-write is involved, so arrivals and polls
// do not queue up behind each other on one cache line as they do with a shared counter (measured: 64 workgroups
// polling a counter with atomics took ~20 us per barrier).  The wait is bounded (see the kernel's comment).
__device__ __forceinline__ bool xcd_barrier(unsigned* slots, int rank, unsigned& epoch, int n_group, int* flags,
                                            unsigned spin_limit, int* host_flags) {
  __shared__ int ok_s;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // this thread's stores have reached the L2
  __syncthreads();
  epoch += 1;
  if (threadIdx.x < 64) {
    if (threadIdx.x == 0) slots[rank] = epoch;
    int ok = 1;
    unsigned spins = 0;
    const int lane = threadIdx.x;
    for (;;) {
      const unsigned v = lane < n_group ? __hip_atomic_load(slots + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : epoch;
      if (__all((int)(v - epoch) >= 0)) break;
      __builtin_amdgcn_s_sleep(JM_SLEEP);
      if (++spins > spin_limit ||
          ((spins & 255) == 0 && (__hip_atomic_load(flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 6))) {
        if (lane == 0) {
          __hip_atomic_fetch_or(flags, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_fetch_or(host_flags, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        ok = 0;
        break;
      }
    }
    if (lane == 0) ok_s = ok;
  }
  __syncthreads();
  return ok_s != 0;
}

// (second launch bound = waves per SIMD: two workgroups of 8 waves per compute unit, i.e. at most 128 registers)
template <typename T>
__global__ __launch_bounds__(NW * 64, 4) void xcd_sampler_kernel(PersistArgs p) {
  __shared__ float part[NW][TILE][TILE + 1];
  __shared__ int rows_s[XCD_MAX_ROWS];
  __shared__ int wave_total[NW];
  __shared__ int xcc_s, rank_s, unconverged_s;
  constexpr int NT = NW * 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Which XCD this workgroup runs on is read from the hardware; its rank among the XCD's workgroups is the order
  // of arrival at a counter only they touch.  The dispatcher deals workgroups round-robin over the XCDs, so each is
  // expected to receive gridDim / 8 of them: a surplus workgroup backs out here (flag 4), a missing one makes the
  // first barrier's bounded wait run out (flag 2); either way the whole grid drains and the host falls back.
  const int n_group = gridDim.x / XCDS;
  if (threadIdx.x == 0) {
    unsigned id;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
    id &= 0xf;
    xcc_s = (int)id;
    unconverged_s = 0;
    rank_s = id < XCDS ? (int)(__hip_atomic_fetch_add(p.bar + (size_t)(XCDS + id) * XCD_LINE, 1u, __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_WORKGROUP) - p.reg_base)
                       : n_group;
  }
  __syncthreads();
  const int group = xcc_s, rank = rank_s;
  if (group >= XCDS || rank < 0 || rank >= n_group) {
    if (threadIdx.x == 0) {
      __hip_atomic_fetch_or(p.flags, 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_or(p.host_report + 64, 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    return;
  }
  const int N = p.N, D = p.D, L = p.L;
  const int per = (N + XCDS - 1) / XCDS;                 // <= XCD_MAX_ROWS (host)
  const int first = group * per, count = max(0, min(per, N - first));
  int* report = p.host_report + group * 8;
  if (count == 0) {                      // (barriers are per XCD: nobody waits for this one)
    if (rank == 0 && threadIdx.x == 0) {
      for (int i = 0; i < 5; ++i) __hip_atomic_store(report + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(report + 5, p.call_id, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    return;
  }
  unsigned* slots = p.bar + (size_t)group * XCD_LINE;
  unsigned* epoch_word = p.bar + (size_t)2 * XCDS * XCD_LINE + group * 32;     // (a cache line per XCD)
  unsigned epoch = *epoch_word;          // where this XCD's previous call stopped counting its barriers

  // x = x_init (or zeros) and its network encoding, for this XCD's samples
  for (size_t i = (size_t)rank * NT + threadIdx.x; i < (size_t)count * D; i += (size_t)n_group * NT) {
    const int n = first + (int)(i / D), t = (int)(i % D);
    const uint8_t v = p.x_init ? p.x_init[(size_t)n * D + t] : 0;
    p.x[(size_t)n * D + t] = v;
    ((T*)p.enc)[frag_offset<T>(n, t, p.enc_chunks)] = Elem<T>::from_f32((float)v);
  }
  if (rank == 0) {
    for (int i = threadIdx.x; i < count; i += NT) {
      p.iters[first + i] = 0;
      p.changed[(size_t)(first + i) * CHG] = 0;
      p.changed[(size_t)(p.n_pad + first + i) * CHG] = 0;
    }
  }
  if (!xcd_barrier(slots, rank, epoch, n_group, p.flags, p.spin_limit, p.host_report + 64)) return;

  long long n_passes = 0, n_sample_passes = 0;
  int parity = 0;
  const bool gs = p.block < D;
  for (int a0 = 0; a0 < D; a0 += p.block) {
    const int b0 = min(a0 + p.block, D);          // block = 0-based positions [a0, b0)
    // entries past the active count are read as sample ids too (their results are discarded)
    for (int i = threadIdx.x; i < XCD_MAX_ROWS; i += NT) rows_s[i] = first + (i < count ? i : 0);
    int n_rows = count;
    __syncthreads();
    const int cap = gs ? (b0 - a0) : p.cap;
    for (int k = 1; k <= cap && n_rows > 0; ++k) {
      const int row_tiles = (n_rows + TILE - 1) / TILE;
      int* changed = p.changed + (size_t)parity * p.n_pad * CHG;
      int in_limit = gs ? b0 - 1 : -1;
      for (int l = 0; l < L; ++l) {
        const PersistLayer& ly = p.layer[l];
        LayerArgs a = {};
        a.A = l == 0 ? p.enc : p.layer[l - 1].out;
        a.W = ly.W;
        a.k_chunks = ly.k_chunks;
        a.bias = ly.bias;
        a.tile_kend = ly.tile_kend;
        a.k_cap = ly.in_pad;
        if (in_limit >= 0) a.k_cap = min(ly.in_pad, (in_limit + 2 * Elem<T>::EPL - 1) / (2 * Elem<T>::EPL) * (2 * Elem<T>::EPL));
        a.n_rows = N;
        a.out = ly.out;
        a.out_chunks = ly.out_chunks;
        a.n_cols = ly.out_dim;
        int tiles = ly.n_tiles;
        if (gs) {
          const int lim = ly.cnt_lt[b0];
          tiles = min(tiles, (lim + TILE - 1) / TILE);
          in_limit = lim;
        }
        for (int item = rank; item < tiles * row_tiles; item += n_group) {
          compute_tile<T, EPI_RELU, true, true>(a, item / row_tiles, (item % row_tiles) * TILE, rows_s, n_rows, part);
          __syncthreads();   // `part` is reused by the next item
        }
        if (!xcd_barrier(slots, rank, epoch, n_group, p.flags, p.spin_limit, p.host_report + 64)) return;
      }
      {
        const PersistLayer& ly = p.layer[L];
        LayerArgs a = {};
        a.A = p.layer[L - 1].out;
        a.W = ly.W;
        a.k_chunks = ly.k_chunks;
        a.bias = ly.bias;
        a.tile_kend = ly.tile_kend;
        a.k_cap = ly.in_pad;
        if (in_limit >= 0) a.k_cap = min(ly.in_pad, (in_limit + 2 * Elem<T>::EPL - 1) / (2 * Elem<T>::EPL) * (2 * Elem<T>::EPL));
        a.tile_begin = a0 / TILE;
        a.n_rows = N;
        a.n_cols = ly.out_dim;
        a.noise = p.noise;
        a.x = p.x;
        a.enc = p.enc;
        a.enc_chunks = p.enc_chunks;
        a.changed = changed;
        a.D = D;
        a.t_lo = a0;
        a.t_hi = b0;
        const int tiles = (b0 + TILE - 1) / TILE - a.tile_begin;
        for (int item = rank; item < tiles * row_tiles; item += n_group) {
          compute_tile<T, EPI_BERNOULLI, true, true>(a, item / row_tiles, (item % row_tiles) * TILE, rows_s, n_rows, part);
          __syncthreads();
        }
        if (!xcd_barrier(slots, rank, epoch, n_group, p.flags, p.spin_limit, p.host_report + 64)) return;
      }
      // stop test and compaction, recomputed identically by every workgroup of the XCD; its first workgroup also keeps
      // the pass counts and clears the counters the pass after next will use
      n_passes += 1;
      n_sample_passes += n_rows;
      const bool last_pass = (k == cap);
      int new_n = 0;
      for (int start = 0; start < n_rows; start += NT) {
        const int rix = start + threadIdx.x;
        int sample = -1;
        bool keep = false;
        if (rix < n_rows) {
          sample = rows_s[rix];
          // (whatever other compute units wrote is read past this unit's L1: device-scope loads)
          const int c = __hip_atomic_load(&changed[(size_t)sample * CHG], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          keep = (c > 0) && !last_pass;
          if (rank == 0) {
            p.iters[sample] = __hip_atomic_load(&p.iters[sample], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
            if (c > 0 && last_pass && p.flag_unconverged) unconverged_s = 1;     // (every writer stores 1)
          }
        }
        const unsigned long long mask = __ballot(keep);
        const int before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_total[wave] = __popcll(mask);
        __syncthreads();
        int off = new_n;
        for (int w = 0; w < wave; ++w) off += wave_total[w];
        if (keep) rows_s[off + before] = sample;
        for (int w = 0; w < NW; ++w) new_n += wave_total[w];
        __syncthreads();
      }
      if (rank == 0) {
        int* other = p.changed + (size_t)(parity ^ 1) * p.n_pad * CHG;
        for (int i = threadIdx.x; i < count; i += NT) other[(size_t)(first + i) * CHG] = 0;
      }
      n_rows = new_n;
      parity ^= 1;
    }
  }
  // The XCD's first workgroup reports.  Its own stores (pass counts) and, through the last barrier, everybody
  // else's (symbols) have reached the L2; the release store of the call's id orders the report words before it.
  if (rank == 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
      *epoch_word = epoch;
      __hip_atomic_store(report + 0, (int)(n_passes & 0xffffffff), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(report + 1, (int)(n_passes >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(report + 2, (int)(n_sample_passes & 0xffffffff), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(report + 3, (int)(n_sample_passes >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(report + 4, unconverged_s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(report + 5, p.call_id, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Output layer of a 256-class categorical model with the Gumbel-max draw fused in: the logits never
// leave the registers.
//
// A workgroup owns ONE position t and up to 64 active samples; it streams the 256 weight rows of t
// exactly once (this layer is the model's HBM stream: 2 GiB dense for D = 1024, K = 4096, of which the
// degree-sorted prefix structure lets it skip about half).  Each of the 4 waves owns 64 classes
// (two 32-row weight tiles) against both 32-sample tiles: 4 accumulator tiles, no split of K, so the
// sum order is fixed.  The MFMA takes the WEIGHTS as its row operand: an accumulator lane then holds
// 16 classes of one sample, the noise comes in 16-byte loads, and the 256-way argmax is 32 in-register
// compares, one exchange between the half-waves and a 4-entry combine through LDS.  (With the samples as row
// operand a lane holds one class of 16 samples and reads the noise 4 bytes at a time, whole 128-byte lines per
// half-wave: measured 1.5 TB/s on the noise stream against 4.2 TB/s for the 16-byte pattern.)  Positions with
// the longest visible prefix are scheduled first.
// ------------------------------------------------------------------------------------------------
constexpr int CAT_C = 256;
constexpr int CAT_WAVES = 4;
constexpr int CAT_PD = 2;

struct CatArgs {
  const void* A;         // last hidden layer's activations (fragment-major, k_chunks chunks)
  const void* W;         // output weights, rows t*256 + c (fragment-major)
  int k_chunks;
  const float* bias;     // [D*256]
  const int* tile_kend;  // per 32-row tile; the 8 tiles of a position share one value
  int k_cap;
  const int* rows;
  const int* n_rows_ptr;
  int n_rows;
  const float* noise;    // g[sample, D, 256]
  uint8_t* x;
  void* enc;
  int enc_chunks;
  int* changed;
  int D;
  int t_lo, t_hi;        // positions whose symbol is re-drawn
  int t_begin, n_pos;    // positions this launch evaluates
  int pair_tiles;        // sample tiles of 64 this launch covers
  // Frozen positions: if no position below t changed in the previous pass (for any sample that is still active),
  // position t reads the inputs it read then and draws the symbol it drew then (its noise is fixed): the pass need
  // not evaluate it -- Proposition 1's frozen prefix, measured instead of bounded.  *t_first_ptr = first position
  // this pass evaluates (NULL: all); first_changed = where it records the lowest position it changes (NULL: nowhere).
  const int* t_first_ptr;
  int* first_changed;
  RetireArgs retire;
};

template <typename T, int CNT, bool TWO>
__device__ __forceinline__ void cat_group(const uint4* W0, const uint4* W1, const uint4* A0, const uint4* A1, int c0,
                                          f32x16 (&acc)[2][2]) {
  uint4 w0[CNT][4], w1[CNT][4], a0[CNT][4], a1[CNT][4];
#pragma unroll
  for (int p = 0; p < CNT; ++p) {
    const size_t o = (size_t)(c0 + p) * 256;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      w0[p][s] = load_stream16(W0 + o + s * 64);
      w1[p][s] = load_stream16(W1 + o + s * 64);
      a0[p][s] = A0[o + s * 64];
      if (TWO) a1[p][s] = A1[o + s * 64];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int p = 0; p < CNT; ++p) {
    mfma_chunk<T>(w0[p], a0[p], acc[0][0]);
    mfma_chunk<T>(w1[p], a0[p], acc[1][0]);
    if (TWO) {
      mfma_chunk<T>(w0[p], a1[p], acc[0][1]);
      mfma_chunk<T>(w1[p], a1[p], acc[1][1]);
    }
  }
}

template <typename T, bool TWO>
__device__ __forceinline__ void cat_stream(const uint4* W0, const uint4* W1, const uint4* A0, const uint4* A1,
                                           int n_chunks, f32x16 (&acc)[2][2]) {
  int c = 0;
  for (; c + CAT_PD <= n_chunks; c += CAT_PD) cat_group<T, CAT_PD, TWO>(W0, W1, A0, A1, c, acc);
  if (c < n_chunks) cat_group<T, 1, TWO>(W0, W1, A0, A1, c, acc);
}

template <typename T>
__global__ __launch_bounds__(CAT_WAVES * 64) void categorical_output_kernel(CatArgs a) {
  static_assert(CAT_PD == 2, "the remainder handling assumes a prefetch depth of 2");
  constexpr int KC = 2 * Elem<T>::EPL;
  __shared__ float sm_val[CAT_WAVES][64];
  __shared__ int sm_idx[CAT_WAVES][64];
  const int n_rows = a.n_rows_ptr ? *a.n_rows_ptr : a.n_rows;
  const int t_first = a.t_first_ptr ? *a.t_first_ptr : 0;
  const int pos_i = blockIdx.x / a.pair_tiles, pair = blockIdx.x % a.pair_tiles;
  const int t = a.t_begin + a.n_pos - 1 - pos_i;
  const int row0 = pair * 64;
  if (row0 < n_rows && t >= t_first) {   // (uniform per workgroup)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, h = lane >> 5;
    const bool two = row0 + 32 < n_rows;
    const int n0 = a.rows ? a.rows[row0 + r] : (row0 + r < a.n_rows ? row0 + r : 0);
    const int n1 = a.rows ? a.rows[row0 + 32 + r] : (row0 + 32 + r < a.n_rows ? row0 + 32 + r : 0);
    int k_end = a.tile_kend[t * (CAT_C / TILE)];
    if (k_end > a.k_cap) k_end = a.k_cap;
    const int n_chunks = (k_end + KC - 1) / KC;
    const size_t group = (size_t)a.k_chunks * 256;
    const uint4* W0 = (const uint4*)a.W + (size_t)(t * (CAT_C / TILE) + wave * 2) * group + h * 32 + r;
    const uint4* W1 = W0 + group;
    const uint4* A0 = (const uint4*)a.A + (size_t)(n0 >> 5) * group + h * 32 + (n0 & 31);
    const uint4* A1 = (const uint4*)a.A + (size_t)(n1 >> 5) * group + h * 32 + (n1 & 31);

    f32x16 acc[2][2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[q][j][i] = 0.f;
    if (two)
      cat_stream<T, true>(W0, W1, A0, A1, n_chunks, acc);
    else
      cat_stream<T, false>(W0, W1, A0, A1, n_chunks, acc);

    // acc[q][j][i]: class (wave*2 + q)*32 + 8*(i/4) + 4*h + i%4 of sample tile j's row r
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (j == 0 || two) {
        const int sample = j ? n1 : n0;
        const float* gp = a.noise + ((size_t)sample * a.D + t) * CAT_C;
        const float* bp = a.bias + (size_t)t * CAT_C;
        float best = -INFINITY;
        int best_c = 0x7fffffff;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const int cb = (wave * 2 + q) * 32 + 8 * i4 + 4 * h;
            const float4 gv = *(const float4*)(gp + cb);
            const float4 bv = *(const float4*)(bp + cb);
            const float v0 = (acc[q][j][i4 * 4 + 0] + bv.x) + gv.x;
            const float v1 = (acc[q][j][i4 * 4 + 1] + bv.y) + gv.y;
            const float v2 = (acc[q][j][i4 * 4 + 2] + bv.z) + gv.z;
            const float v3 = (acc[q][j][i4 * 4 + 3] + bv.w) + gv.w;
            // classes are visited in increasing order, so a strict compare keeps the lowest index of a tie
            if (v0 > best) { best = v0; best_c = cb; }
            if (v1 > best) { best = v1; best_c = cb + 1; }
            if (v2 > best) { best = v2; best_c = cb + 2; }
            if (v3 > best) { best = v3; best_c = cb + 3; }
          }
        }
        const float ob = __shfl_xor(best, 32);
        const int oc = __shfl_xor(best_c, 32);
        if (ob > best || (ob == best && oc < best_c)) { best = ob; best_c = oc; }
        if (h == 0) {
          sm_val[wave][32 * j + r] = best;
          sm_idx[wave][32 * j + r] = best_c;
        }
      }
    }
    __syncthreads();
    if (threadIdx.x < 64) {   // (wave 0: one lane per sample row of the pair)
      const int sl = threadIdx.x;
      const bool redraw = row0 + sl < n_rows && t >= a.t_lo && t < a.t_hi;
      bool differs = false;
      int sample = 0;
      if (redraw) {
        float best = sm_val[0][sl];
        int best_c = sm_idx[0][sl];
#pragma unroll
        for (int w = 1; w < CAT_WAVES; ++w)
          if (sm_val[w][sl] > best) { best = sm_val[w][sl]; best_c = sm_idx[w][sl]; }   // waves hold increasing classes
        sample = a.rows ? a.rows[row0 + sl] : row0 + sl;
        const size_t idx = (size_t)sample * a.D + t;
        const uint8_t xn = (uint8_t)best_c;
        differs = xn != a.x[idx];
        if (differs) {
          a.x[idx] = xn;
          if (a.enc)
            ((T*)a.enc)[frag_offset<T>(sample, t, a.enc_chunks)] =
                Elem<T>::from_f32(((float)xn - 128.0f) * (1.0f / 128.0f));
        }
      }
      if (differs) count_changed(&a.changed[(size_t)sample * CHG], 1);
      if (a.first_changed && __ballot(differs) != 0 && threadIdx.x == 0) {
        // (returning atomic: performed before this workgroup reports in, like the counters above)
        const int old = __hip_atomic_fetch_min(a.first_changed, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("" ::"v"(old));
      }
    }
  }
  if (a.retire.enabled) finish_pass(a.retire, gridDim.x);
}

__global__ void conv_reset_window_kernel(int* dirty_lo, int* first_changed, int n, int* win_done,
                                         unsigned long long* rows_stat) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    dirty_lo[i] = 0;
    first_changed[(size_t)i * CHG] = 0x7fffffff;
  }
  if (i == 0) {
    *win_done = 0;
    *rows_stat = 0;
  }
}

// ------------------------------------------------------------------------------------------------
// Masked convolutional model (images of width 32: one row of pixels is one 32-row operand group).
// Activations are fragment-major with rows = pixels ((n*H + y)*32 + x) and K = feature channels.
// ------------------------------------------------------------------------------------------------
constexpr int CONV_MAX_K = 7;
constexpr int CONV_ROWS = 4;             // image rows per workgroup of the k x k layers

// Row window of a pass over the convolutional network.  The activations of every layer persist between passes
// (one buffer per layer).  A state only depends on pixels above it and to its left, so as long as no symbol of
// rows < d changed since they were computed, the activation rows < d of every layer are still those of the
// current symbols: a pass only has to recompute rows d .. row_hi, where row_hi is the last row whose logits it
// needs.  dirty_lo[n] holds d for image n and is maintained by the tail of the sampling kernel.
struct ConvWindow {
  const int* dirty_lo;   // NULL: recompute every row up to row_hi
  int row_hi;
  const int* row_hi_of;  // per image instead of the common row_hi (NULL: row_hi).  Algorithm 2 gives every block a
                         // copy of the image of its own, and each copy only needs the rows of its block's current state
};
__device__ __forceinline__ bool conv_rows_active(const ConvWindow& w, int n, int y0, int rows) {
  const int lo = w.dirty_lo ? w.dirty_lo[n] : 0;
  const int hi = w.row_hi_of ? w.row_hi_of[n] : w.row_hi;
  return y0 + rows > lo && y0 <= hi;
}

struct ConvFirstArgs {
  ConvWindow win;
  const uint8_t* x;      // symbols [N, H, 32, 3]
  const void* w;         // masked weights as a [F x K0] matrix, fragment-major; K index = tap * 3 + colour with the
                         // visible taps in row-major order (tap = (dy + MID) * KS + dx + MID), zero beyond 3 * n_taps
  const float* bias;     // [F]
  void* out;             // activations, fragment-major, out_chunks chunks
  int out_chunks;
  int N, H;
};

// First layer (3 input colours, type A) as a small GEMM on the matrix cores: the inputs (v - 128) / 128 are
// exact in bf16, so nothing is lost against fp32 FMAs.  A workgroup owns one row of 32 pixels; wave w owns
// channel tile w (F / 32 waves).  The MID + 1 symbol rows the pixels can see are copied to LDS as bytes (zero
// padded left and right); within one kernel row the K index tap * 3 + colour runs along consecutive bytes of
// that copy, so the 32 x K0 operand is built in LDS, in fragment order, with one byte read per element.
template <typename T, int FT, int KS>
__global__ __launch_bounds__(FT * 64) void conv_first_kernel(ConvFirstArgs a) {
  constexpr int MID = KS / 2, NT = MID * KS + MID + 1, K_LIVE = NT * 3;
  constexpr int KC = 2 * Elem<T>::EPL;
  constexpr int K0_CHUNKS = (K_LIVE + KC - 1) / KC, K0 = K0_CHUNKS * KC;
  constexpr int ROWB = (32 + 2 * MID) * 3;          // bytes per padded symbol row
  constexpr int NTHREADS = FT * 64;
  __shared__ uint8_t xt[(MID + 1) * ROWB + 16];
  __shared__ __align__(16) T a_lds[32 * K0];        // one row group of the operand, fragment-major
  const int g = blockIdx.x;                         // group = row of pixels (n, y)
  const int n = g / a.H, y = g % a.H;
  if (!conv_rows_active(a.win, n, y, 1)) return;    // (uniform over the workgroup)
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;

  // this wave's weights: K0_CHUNKS chunks of channel tile `wave`
  const uint4* Wp = (const uint4*)a.w + (size_t)wave * K0_CHUNKS * 256 + h * 32 + r;
  uint4 wf[K0_CHUNKS][4];
#pragma unroll
  for (int c = 0; c < K0_CHUNKS; ++c)
#pragma unroll
    for (int s = 0; s < 4; ++s) wf[c][s] = Wp[(size_t)c * 256 + s * 64];
  // the weights are the MFMA's row operand, so lane (r, h) ends up with pixel r and the runs of four channels
  // 8 q + 4 h .. + 3 of its channel tile: its bias values are requested now
  const int ch0 = wave * TILE + 4 * h;
  float4 bias4[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) bias4[q] = *(const float4*)(a.bias + ch0 + 8 * q);

  // symbol rows y - MID .. y with MID pixels of padding on both sides
  for (int e = tid; e < (MID + 1) * ROWB; e += NTHREADS) {
    const int row = e / ROWB, col = e % ROWB;       // col = (pixel + MID) * 3 + colour
    const int yy = y - MID + row, xb = col - 3 * MID;
    const bool ok = yy >= 0 && xb >= 0 && xb < 96;
    const uint8_t v = a.x[((size_t)n * a.H + (ok ? yy : 0)) * 96 + (ok ? xb : 0)];
    xt[e] = ok ? v : (uint8_t)128;                  // 128 encodes the value 0
  }
  __syncthreads();
  // operand element (pixel, k): kernel row dyi = k / (3 KS), byte (pixel * 3 + k % (3 KS)) of that padded row
  for (int e = tid; e < 32 * K0; e += NTHREADS) {
    const int px = e & 31, k = e >> 5;
    float v = 0.f;
    if (k < K_LIVE) {
      const int dyi = k / (3 * KS), rem = k - dyi * 3 * KS;
      v = ((float)xt[dyi * ROWB + px * 3 + rem] - 128.0f) * (1.0f / 128.0f);
    }
    a_lds[frag_offset<T>(px, k, K0_CHUNKS)] = Elem<T>::from_f32(v);
  }
  __syncthreads();

  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const uint4* Ap = (const uint4*)a_lds + h * 32 + r;
#pragma unroll
  for (int c = 0; c < K0_CHUNKS; ++c) {
    uint4 af[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) af[s] = Ap[c * 256 + s * 64];
    mfma_chunk<T>(wf[c], af, acc);                  // (channels = rows of the result)
  }

  // acc[4 q + c] = channel ch0 + 8 q + c of pixel r: four consecutive channels are half a 16-byte piece (bf16) or a
  // whole one (fp32) of the fragment-major activations, stored straight from the registers
  const size_t out_row = frag_row_offset<T>(g * 32 + r, a.out_chunks);
#pragma unroll
  for (int q = 0; q < 4; ++q)
    store_quad<T>((T*)a.out + (out_row + frag_col_offset<T>(ch0 + 8 * q)), fmaxf(acc[4 * q + 0] + bias4[q].x, 0.f),
                  fmaxf(acc[4 * q + 1] + bias4[q].y, 0.f), fmaxf(acc[4 * q + 2] + bias4[q].z, 0.f),
                  fmaxf(acc[4 * q + 3] + bias4[q].w, 0.f));
}

struct ConvLayerArgs {
  ConvWindow win;
  const void* in;        // activations of the previous layer (fragment-major, F channels)
  const void* w;         // masked weights as a [F x (n_taps * F)] matrix, tap-major K, fragment-major
  const float* bias;
  void* out;
  int N, H;
};

// k x k masked convolution F -> F as an implicit GEMM over the visible taps (rows above, and the same row up
// to the centre).  A workgroup owns WG_ROWS image rows of one image and all F output channels; a wave owns one
// 32-channel tile and RW of those rows (4 waves: F = 128 -> RW = WG_ROWS, F = 64 -> RW = WG_ROWS / 2).
//
// The input rows the workgroup needs (its own and MID = (k-1)/2 rows above; taps below are masked out) are
// copied to LDS once, each 32-pixel run padded with MID zero entries on both sides, so the operand of tap
// (dy, dx) is the same LDS data read at a row offset and an entry offset: no im2col buffer, no lane masks.
// The loop runs over (dx, K chunk).  For one such step the weights of all visible dy (2 or 3 fragments of
// 32 channels x 128 B) sit in registers while the wave walks down its RW + MID input rows: every input
// fragment read from LDS feeds up to MID + 1 output rows (dy = input row - output row), which halves the LDS
// traffic per MFMA, and a step is long enough (up to 12 x 4 MFMAs) to cover the L2 latency of the next
// step's weights, which are requested at its start.
template <typename T, int FT, int KS, int WG_ROWS>
__global__ __launch_bounds__(256) void conv_layer_kernel(ConvLayerArgs a) {
  constexpr int MID = KS / 2;
  constexpr int NDY = MID + 1;
  constexpr int KCH = FT * 32 / (2 * Elem<T>::EPL);     // K chunks per tap (= chunks per activation row group)
  constexpr int ROW_SPLIT = 4 / FT;                     // waves along the rows
  constexpr int RW = WG_ROWS / ROW_SPLIT;               // output rows per wave
  static_assert(RW >= 1 && RW * ROW_SPLIT == WG_ROWS, "rows must divide among the waves");
  constexpr int PADW = 32 + 2 * MID;                    // entries per padded 32-pixel run
  constexpr int ROWBLK = KCH * 8 * PADW;                // uint4 per image row in LDS
  constexpr int LDS_ROWS = WG_ROWS + MID;
  extern __shared__ uint4 conv_lds[];                   // [LDS_ROWS][KCH][slot*2 + half][PADW]
  const int tiles_y = (a.H + WG_ROWS - 1) / WG_ROWS;
  const int n = blockIdx.x / tiles_y, y0 = (blockIdx.x % tiles_y) * WG_ROWS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int ct = wave % FT;                             // channel tile of this wave
  const int wrow = (wave / FT) * RW;                    // its first output row within the workgroup's rows
  if (!conv_rows_active(a.win, n, y0, WG_ROWS)) return; // (uniform over the workgroup)

  // weights: row group = output channel tile, chunk index = tap * KCH + c, tap = (dy + MID) * KS + (dx + MID)
  const size_t wgroup = (size_t)(MID * KS + MID + 1) * KCH * 256;
  const uint4* Wp = (const uint4*)a.w + (size_t)ct * wgroup + h * 32 + r;
  // Three weight buffers: step p uses buffer p % 3; at its start the fragments of step p + 2 are requested into the
  // buffer step p - 1 has just finished with, so a fragment has two whole steps (> 1 us) to arrive from L2.
  constexpr int NBUF = 3;
  uint4 wbuf[NBUF][NDY][4];
  auto load_weight_frag = [&](int it, auto D, uint4 (&dst)[4]) {
    constexpr int dyi = decltype(D)::value;
    const int dxi = it / KCH, c = it - dxi * KCH;
    const uint4* p = Wp + (size_t)((dyi * KS + dxi) * KCH + c) * 256;
#pragma unroll
    for (int s = 0; s < 4; ++s) dst[s] = p[s * 64];
  };
  // Steps (dx, chunk) come in two runs: dx <= 0 (MID + 1 visible dy each) and dx > 0 (MID visible dy), each a
  // loop with a single straight-line body.  Within a run the workgroups start at different steps: all of them
  // read the same few hundred KB of weights, and in lock-step they would all ask the same L2 channel for the
  // same lines at the same time.  The starting step fixes the order of the fp32 additions, so it is taken from
  // the rows' place in the image alone: an image's activations are the same bits wherever it sits in the batch
  // (Algorithm 2 evaluates copies of an image at other batch positions and must reach the same fixed point).
  constexpr int N_A = (MID + 1) * KCH, N_B = MID * KCH, N_IT = N_A + N_B;
  const int rot_a = (y0 / WG_ROWS) % N_A, rot_b = (y0 / WG_ROWS) % N_B;
  auto step_of = [&](int p) {               // p-th step of this workgroup -> it = dxi * KCH + c
    if (p < N_A) { const int q = p + rot_a; return q < N_A ? q : q - N_A; }
    const int q = p - N_A + rot_b;
    return N_A + (q < N_B ? q : q - N_B);
  };
  // entry of pixel r + dx in the padded run of (input row wrow + j, chunk c, slot s, half h)
  auto frag_ptr = [&](int it) {
    const int dxi = it / KCH, c = it - dxi * KCH;
    return conv_lds + ((size_t)(wrow * KCH + c) * 8 + h) * PADW + r + dxi;
  };
  JM_TSTAMP(0, 0);
  static_for<2>([&](auto P) {
    constexpr int p = decltype(P)::value;
    if constexpr (p < N_IT) {
      const int it = step_of(p);
      static_for<NDY>([&](auto D) {
        if (decltype(D)::value < MID || it < N_A) load_weight_frag(it, D, wbuf[p][decltype(D)::value]);
      });
    }
  });
  // the weights are the MFMA's row operand, so lane (r, h) ends up with pixel r and the runs of four channels
  // 8 g + 4 h .. + 3 of its channel tile: its bias values are requested now
  const int ch0 = ct * TILE + 4 * h;
  float4 bias4[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) bias4[g] = *(const float4*)(a.bias + ch0 + 8 * g);

  // input rows y0 - MID .. y0 + WG_ROWS - 1 -> LDS (rows outside the image and the pads are zero); the loads of
  // a batch are all issued before the first store so that their latencies overlap
  constexpr int FILL = LDS_ROWS * KCH;                  // 16-byte pieces per thread
  constexpr int FILL_BATCH = FILL < 12 ? FILL : 12;
  static_for<(FILL + FILL_BATCH - 1) / FILL_BATCH>([&](auto B) {
    constexpr int b0 = decltype(B)::value * FILL_BATCH;
    constexpr int cnt = FILL - b0 < FILL_BATCH ? FILL - b0 : FILL_BATCH;
    uint4 v[cnt];
#pragma unroll
    for (int i = 0; i < cnt; ++i) {
      const int e = tid + (b0 + i) * 256;
      const int lr = e / (KCH * 256), off = e % (KCH * 256);     // off = (c*8 + slot*2 + half)*32 + pixel
      const int y = y0 - MID + lr;
      const bool ok = y >= 0 && y < a.H;                          // (clamped address: a load without a branch)
      v[i] = ((const uint4*)a.in)[((size_t)n * a.H + (ok ? y : 0)) * (KCH * 256) + off];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < cnt; ++i) {
      const int e = tid + (b0 + i) * 256;
      const int lr = e / (KCH * 256), off = e % (KCH * 256);
      const int y = y0 - MID + lr;
      const uint32_t keep = (y >= 0 && y < a.H) ? 0xffffffffu : 0u;
      conv_lds[(lr * KCH * 8 + (off >> 5)) * PADW + MID + (off & 31)] =
          make_uint4(v[i].x & keep, v[i].y & keep, v[i].z & keep, v[i].w & keep);
    }
  });
  for (int e = tid; e < LDS_ROWS * KCH * 8 * 2 * MID; e += 256) {
    const int run = e / (2 * MID), q = e % (2 * MID);
    conv_lds[run * PADW + (q < MID ? q : 32 + q)] = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();
  JM_TSTAMP(1, 0);

  f32x16 acc[RW];
#pragma unroll
  for (int o = 0; o < RW; ++o)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[o][e] = 0.f;

  // A step walks down the wave's input rows j = 0 .. RW + (visible dy) - 2 (LDS row j holds image row
  // y0 + wrow - MID + j): the fragment of row j feeds the output rows o = j - dyi of every visible dy, i.e. up to
  // MID + 1 MFMA groups, and is then dead.  Fragments are read from LDS AHEAD input rows before they are used,
  // through a ring of AHEAD + 1 register sets, continuing across step boundaries, so that the LDS latency is
  // covered by the MFMAs of the rows in between and only AHEAD + 1 fragments are live at a time (holding all
  // RW + MID fragments of a step at once cost 64 registers more and left their reads exposed at every step's
  // start).  A step has NJP row slots, NJ = RW + MID rounded up to a multiple of the ring size, so that slot j
  // always uses register set j % RING; slots without a row do nothing but the reads ahead.
  constexpr int NJ = RW + MID;
  constexpr int AHEAD = 2, RING = AHEAD + 1;
  constexpr int NJP = (NJ + RING - 1) / RING * RING;
  static_assert(NJP >= AHEAD, "a step must have room for the reads ahead");
  uint4 af[RING][4];
  auto read_row = [&](const uint4* base, int j, uint4 (&dst)[4]) {
#pragma unroll
    for (int s = 0; s < 4; ++s) dst[s] = base[(size_t)j * ROWBLK + s * 2 * PADW];
  };
  {
    const uint4* base = frag_ptr(step_of(0));
    static_for<AHEAD>([&](auto J) { read_row(base, decltype(J)::value, af[decltype(J)::value]); });
  }
  // one step: p = its index in this workgroup's order, BUF = p % NBUF
  auto one_step = [&](auto NV, auto BUF, int p) {
    constexpr int n_visible = decltype(NV)::value;             // visible dy of this step
    constexpr int buf = decltype(BUF)::value;
    constexpr int rows_used = RW + n_visible - 1;              // input rows this step reads
    const uint4* base = frag_ptr(step_of(p));
    const uint4* base_next = frag_ptr(step_of(p + 1 < N_IT ? p + 1 : p));
    if (p + 2 < N_IT) {                                        // weights of step p + 2
      const int it2 = step_of(p + 2);
      static_for<NDY>([&](auto D) {
        if (decltype(D)::value < MID || it2 < N_A) load_weight_frag(it2, D, wbuf[(buf + 2) % NBUF][decltype(D)::value]);
      });
    }
    // (the scheduler otherwise sinks every load to just before its first use, to save registers, and the
    // wave then waits out each L2 and LDS latency in turn)
    __builtin_amdgcn_sched_barrier(0);
    static_for<NJP>([&](auto J) {
      constexpr int j = decltype(J)::value;
      constexpr int ja = j + AHEAD;                            // the row read now, used AHEAD slots later
      if constexpr (ja < NJP) {
        if constexpr (ja < rows_used) read_row(base, ja, af[ja % RING]);
      } else {
        read_row(base_next, ja - NJP, af[(ja - NJP) % RING]);  // (rows 0 .. AHEAD-1 exist in every step)
      }
      if constexpr (j < rows_used) {
        static_for<n_visible>([&](auto D) {
          constexpr int dyi = decltype(D)::value, o = j - dyi;  // dy = dyi - MID reads input row j = o + dyi
          if constexpr (o >= 0 && o < RW) mfma_chunk<T>(wbuf[buf][dyi], af[j % RING], acc[o]);   // (channels = rows of the result)
        });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if (p == 0) JM_TSTAMP(2, 0);
    if (p == 4) JM_TSTAMP(3, 0);
  };
  // run A: steps 0 .. N_A-1 (dx <= 0), run B: steps N_A .. N_IT-1 (dx > 0); buffers rotate throughout
  auto run_steps = [&](auto NV, auto PHASE, int p_begin, int p_end) {
    constexpr int ph = decltype(PHASE)::value;
    for (int p = p_begin; p < p_end; p += NBUF) {
      one_step(NV, std::integral_constant<int, ph>{}, p);
      if (p + 1 < p_end) one_step(NV, std::integral_constant<int, (ph + 1) % NBUF>{}, p + 1);
      if (p + 2 < p_end) one_step(NV, std::integral_constant<int, (ph + 2) % NBUF>{}, p + 2);
    }
  };
  run_steps(std::integral_constant<int, NDY>{}, std::integral_constant<int, 0>{}, 0, N_A);
  run_steps(std::integral_constant<int, MID>{}, std::integral_constant<int, N_A % NBUF>{}, N_A, N_IT);
  JM_TSTAMP(4, 0);

  // epilogue: acc[o][4 g + c] = channel ch0 + 8 g + c of pixel r in output row o.  Four consecutive channels are
  // half a 16-byte piece (bf16) or a whole one (fp32) of the fragment-major activations: stored straight from the
  // registers, converted by the hardware (the first version turned every tile through an LDS patch to get
  // 16-byte stores, which took longer than the stores saved).
  uint32_t out_col[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) out_col[g] = frag_col_offset<T>(ch0 + 8 * g);
  static_for<RW>([&](auto O) {
    constexpr int o = decltype(O)::value;
    const int y = y0 + wrow + o;
    if (y < a.H) {
      const size_t out_row = frag_row_offset<T>(((n * a.H) + y) * 32 + r, KCH);
#pragma unroll
      for (int g = 0; g < 4; ++g)
        store_quad<T>((T*)a.out + (out_row + out_col[g]), fmaxf(acc[o][4 * g + 0] + bias4[g].x, 0.f),
                      fmaxf(acc[o][4 * g + 1] + bias4[g].y, 0.f), fmaxf(acc[o][4 * g + 2] + bias4[g].z, 0.f),
                      fmaxf(acc[o][4 * g + 3] + bias4[g].w, 0.f));
    }
  });
  JM_TSTAMP(5, 1);
}

struct ConvHeadArgs {
  const void* A;         // last k x k layer's activations (fragment-major, rows = pixels, F channels)
  const void* W;         // head weights [3*256 x F], rows colour*256 + class (fragment-major)
  const float* bias;     // [3*256]
  const int* tile_kend;  // [3*8] visible K per 32-row weight tile; the 8 tiles of a colour share one value
  const float* noise;    // g[pixel, colour, 256]
  uint8_t* x;            // symbols [pixel, colour]
  int* changed;          // per image: states changed in this pass
  int N, H;
  int state_lo, state_hi;   // states (pixel within its image * 3 + colour) that are re-drawn
  int groups;               // workgroups per colour; workgroup (colour, group) walks rows group, group + groups, ...
  // row window (see ConvWindow); first_changed == NULL: every row is evaluated and nothing is tracked
  int* dirty_lo;
  int* first_changed;
  int* win_done;
  unsigned long long* rows_stat;
  int row_lo, row_hi, first_pass;
  // Algorithm 2 (virtual images, see jacobi_gs_sample): image n draws the ONE state state_one[n] (or none if negative)
  // and reads the noise of image n % noise_images; nothing is counted or tracked.  NULL: the windows above apply.
  const int* state_one;
  int noise_images;
  RetireArgs retire;
};

constexpr int HEAD_BATCH = 16;               // rows a workgroup draws between two of its finishing phases

// 1 x 1 head + Gumbel-max draw + change detection of the convolutional model.  A workgroup is bound to one colour
// and walks rows of 32 pixels (rows group, group + groups, ...); its 4 waves split the 256 classes: wave w keeps the
// weights of classes 64 w .. 64 w + 63 (two 32-class tiles) in registers for the whole launch -- nothing is staged
// in LDS and no barrier stands between the launch and the first MFMA.  The classes are the MFMA's row operand, so
// lane (r, h) holds 16 classes of pixel r per tile: a wave's argmax over its 64 classes is a running
// (value, class) pair per lane plus one exchange between the half-waves.  The four partial results of a row go
// through LDS; every HEAD_BATCH rows (and at the end) the workgroup meets once, picks the winner per pixel, compares
// it with the old symbol and counts the changes.  The noise is the large stream of this launch (100 MB per pass at
// batch 32 against 8 MB of activations); see load_row for how it is fetched.  FT = F / 32.
template <typename T, int FT>
__global__ __launch_bounds__(256) void conv_head_kernel(ConvHeadArgs a) {
  constexpr int KC = 2 * Elem<T>::EPL;
  constexpr int KCH = FT * 32 / KC;
  constexpr int NCT = CAT_C / TILE;                     // class tiles
  constexpr int WT = NCT / 4;                           // class tiles per wave
  constexpr int RR = sizeof(T) == 2 ? 3 : 2;            // rows whose inputs are in flight or in registers
  static_assert(NCT % 4 == 0, "the class tiles are dealt to four waves");
  __shared__ float cand_v[HEAD_BATCH][4][TILE];         // per row of the batch and wave: the wave's best value ...
  __shared__ int cand_c[HEAD_BATCH][4][TILE];           // ... and its class, per pixel
  __shared__ int batch_row[HEAD_BATCH];
  __shared__ uint8_t batch_x[HEAD_BATCH][TILE];         // the rows' old symbols
  const int t = blockIdx.x / a.groups, group = blockIdx.x % a.groups;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int n_rows = a.N * a.H;

  auto row_active = [&](int g) {
    const int n = g / a.H, y = g % a.H;
    if (a.state_one) {
      const int st = a.state_one[n];
      return st >= 0 && st % 3 == t && st / 96 == y;
    }
    if (y * 96 + 93 + t < a.state_lo || y * 96 + t >= a.state_hi) return false;   // no state of this row is drawn
    if (!a.first_changed) return true;
    const int lo = a.first_pass ? a.row_lo : max(a.row_lo, a.dirty_lo[n]);
    return y >= lo && y <= a.row_hi;
  };
  // The workgroup's rows are group, group + stride, ...; which of them are active is decided 64 rows at a time (every
  // wave for itself, all with the same result: nothing these tests read is written before the launch's tail).
  const int stride = a.groups;
  const int g_first = group;
  int chunk = 0;                                        // rows g_first + (64 * chunk + k) * stride, k = 0..63
  auto active_mask = [&](int ch) {                      // (lane k tests row k of the chunk)
    const long long gg = g_first + (long long)(64 * ch + lane) * stride;
    return (unsigned long long)__ballot(gg < n_rows && row_active((int)gg));
  };
  unsigned long long mask = active_mask(0);
  // first active row at or after position k of the current chunk (moves on to later chunks when needed)
  auto next_active = [&](int k) {
    for (;;) {
      const unsigned long long rest = k < 64 ? (mask >> k) << k : 0ull;
      if (rest) return g_first + (64 * chunk + __builtin_ctzll(rest)) * stride;
      if (g_first + (long long)(64 * (chunk + 1)) * stride >= n_rows) return n_rows;
      ++chunk;
      mask = active_mask(chunk);
      k = 0;
    }
  };
  auto slot_of = [&](int gg) { return (gg - g_first) / stride - 64 * chunk; };
  auto row_after = [&](int gg) { return gg < n_rows ? next_active(slot_of(gg) + 1) : n_rows; };
  JM_TSTAMP(0, 0);

  // ---- what stays in registers: the wave's weights and bias
  int k_end = a.tile_kend[t * NCT];
  if (k_end > FT * 32) k_end = FT * 32;
  const int n_chunks = (k_end + KC - 1) / KC;
  const int ct0 = wave * WT;                            // the wave's first class tile
  uint4 wf[WT][KCH][4];
  {
    const uint4* Wsrc = (const uint4*)a.W + ((size_t)t * NCT + ct0) * KCH * 256 + h * 32 + r;
#pragma unroll
    for (int j = 0; j < WT; ++j)
#pragma unroll
      for (int c = 0; c < KCH; ++c)
#pragma unroll
        for (int s = 0; s < 4; ++s) wf[j][c][s] = Wsrc[(size_t)(j * KCH + c) * 256 + s * 64];
  }
  float4 bias4[WT][4];                                  // classes (ct0 + j) * 32 + 8 q + 4 h .. + 3
#pragma unroll
  for (int j = 0; j < WT; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) bias4[j][q] = *(const float4*)(a.bias + t * CAT_C + (ct0 + j) * TILE + 8 * q + 4 * h);

  // ---- a row's inputs: the activations of its 32 pixels (every wave needs all of them) and the wave's share of
  // the noise, both into the same ring slot and requested together, RR rows ahead: loads return in order, so
  // whatever a row needs must not sit behind requests of later rows.  The noise is fetched in the accumulator
  // layout at once: lane (r, h) takes classes 8q + 4h .. + 3 of pixel r for q = 0..3 of each tile, 16 bytes a load
  // (a pixel's 128-byte line of a tile is covered by the four loads of its two lanes and stays in the cache between
  // them: no non-temporal hint here).  Fetching whole lines per group of 8 lanes and turning the tile through an
  // LDS patch reads the stream faster on its own (5.6 against 4.2 TB/s, loads only) but the launch is bound by
  // the dependent work per row, which the patch lengthens: 25.2 us per launch with it, 24.6 without.
  typedef __attribute__((__vector_size__(4 * sizeof(float)))) float vf4;   // (a native vector: stays in registers)
  uint4 af[RR][KCH][4];
  vf4 gz[RR][WT][4];
  uint8_t xo[RR];                                       // old symbol of pixel r (used by wave 0 only)
  auto load_row = [&](int g_row, uint4 (&af_dst)[KCH][4], vf4 (&gz_dst)[WT][4], uint8_t& xo_dst) {
    xo_dst = a.x[((size_t)g_row * 32 + r) * 3 + t];
    const uint4* A0 = (const uint4*)a.A + (size_t)g_row * KCH * 256 + h * 32 + r;
    static_for<KCH>([&](auto C) {
      constexpr int c = decltype(C)::value;
#pragma unroll
      for (int s = 0; s < 4; ++s) af_dst[c][s] = A0[c * 256 + s * 64];
    });
    int g_noise = g_row;
    if (a.state_one) g_noise = ((g_row / a.H) % a.noise_images) * a.H + g_row % a.H;   // (a virtual image: its real image's noise)
    const float* nz = a.noise + ((size_t)(g_noise * 32 + r) * 3 + t) * CAT_C + ct0 * TILE + 4 * h;
    static_for<WT>([&](auto J) {
      constexpr int j = decltype(J)::value;
      static_for<4>([&](auto Q) {
        constexpr int q = decltype(Q)::value;
        gz_dst[j][q] = *(const vf4*)(nz + j * TILE + 8 * q);
      });
    });
  };
  // Active rows go through the slots round-robin, in order; g_slot[s] is the row whose inputs slot s holds
  // (n_rows: none).  One cursor walks the active rows: the next one to request.
  int g_req = next_active(0);
  int g_slot[RR];
  static_for<RR>([&](auto S) {
    constexpr int s = decltype(S)::value;
    g_slot[s] = g_req;
    if (g_req < n_rows) {
      load_row(g_req, af[s], gz[s], xo[s]);
      g_req = row_after(g_req);
    }
  });
  JM_TSTAMP(1, 0);
  int sink = 0;                                         // old values of the counter atomics (see below)
  int n_batch = 0;                                      // rows drawn since the last finishing phase

  // ---- finishing phase: winner per pixel over the four waves, comparison with the old symbol, counters
  auto finish_batch = [&]() {
    __syncthreads();
    for (int b = tid >> 5; b < n_batch; b += 8) {       // (half-waves take rows; both halves of a wave run the same trips
                                                        //  or the upper half sits one out: no barrier inside)
      const int g = batch_row[b];
      const int n = g / a.H, y = g % a.H;
      float best = cand_v[b][0][r];
      int best_c = cand_c[b][0][r];
#pragma unroll
      for (int w = 1; w < 4; ++w) {                     // (classes ascend with the wave: a strict compare keeps the lowest)
        const float v = cand_v[b][w][r];
        if (v > best) { best = v; best_c = cand_c[b][w][r]; }
      }
      const int st = (y * 32 + r) * 3 + t;
      bool differs = false;
      if (a.state_one ? st == a.state_one[n] : (st >= a.state_lo && st < a.state_hi)) {
        const uint8_t xn = (uint8_t)best_c;
        differs = xn != batch_x[b][r];
        if (differs) a.x[((size_t)g * 32 + r) * 3 + t] = xn;
      }
      const unsigned long long both = __ballot(differs);
      const unsigned changed_mask = h ? (unsigned)(both >> 32) : (unsigned)both;
      if (r == 0 && changed_mask != 0 && !a.state_one) {
        // returning atomics, so that "the value came back" means "performed"; the values are only consumed
        // after the loop (before the tail counters)
        sink += __hip_atomic_fetch_add(&a.changed[(size_t)n * CHG], __popc(changed_mask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (a.first_changed)
          sink += __hip_atomic_fetch_min(&a.first_changed[(size_t)n * CHG], y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    __syncthreads();
    n_batch = 0;
  };

  // ---- the row loop, with the number of visible K chunks as a compile-time constant (a colour sees its own and
  // the earlier colours' channel groups only; a run-time test per chunk would cut the row into scheduling regions)
  auto row_loop = [&](auto NCH) {
  constexpr int nch = decltype(NCH)::value;
  // one row out of ring slot S
  auto draw_row = [&](auto S) {
    constexpr int s = decltype(S)::value;
    float best = -INFINITY;
    int best_c = 0;
    static_for<WT>([&](auto J) {
      constexpr int j = decltype(J)::value;
      f32x16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
      static_for<KCH>([&](auto C) {
        constexpr int c = decltype(C)::value;
        if constexpr (c < nch) mfma_chunk<T>(wf[j][c], af[s][c], acc);
      });
      // acc[4q + i]: class (ct0 + j)*32 + 8q + 4h + i of pixel r; classes ascend along (j, q, i), so a strict compare
      // keeps the lowest class of a tie
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int cb = (ct0 + j) * TILE + 8 * q + 4 * h;
        const float4 bv = bias4[j][q];
        const vf4 gv = gz[s][j][q];
        const float v0 = (acc[4 * q + 0] + bv.x) + gv[0];
        const float v1 = (acc[4 * q + 1] + bv.y) + gv[1];
        const float v2 = (acc[4 * q + 2] + bv.z) + gv[2];
        const float v3 = (acc[4 * q + 3] + bv.w) + gv[3];
        if (v0 > best) { best = v0; best_c = cb; }
        if (v1 > best) { best = v1; best_c = cb + 1; }
        if (v2 > best) { best = v2; best_c = cb + 2; }
        if (v3 > best) { best = v3; best_c = cb + 3; }
      }
    });
    {
      const float ob = __shfl_xor(best, 32);
      const int oc = __shfl_xor(best_c, 32);
      if (ob > best || (ob == best && oc < best_c)) { best = ob; best_c = oc; }
    }
    if (h == 0) {
      cand_v[n_batch][wave][r] = best;
      cand_c[n_batch][wave][r] = best_c;
    }
    if (tid == 0) batch_row[n_batch] = g_slot[s];
    if (tid < TILE) batch_x[n_batch][r] = xo[s];
    ++n_batch;
    // the slot is free: the row RR places on goes into it
    g_slot[s] = g_req;
    if (g_req < n_rows) {
      load_row(g_req, af[s], gz[s], xo[s]);
      g_req = row_after(g_req);
    }
    __builtin_amdgcn_sched_barrier(0);                  // (keeps the requests here instead of at their use much later)
    if (n_batch == HEAD_BATCH) finish_batch();
  };
  while (g_slot[0] < n_rows) {                          // (uniform over the workgroup)
    static_for<RR>([&](auto S) {
      if (g_slot[decltype(S)::value] < n_rows) draw_row(S);
    });
  }
  };
  static_for<KCH + 1>([&](auto NCH) {
    if (n_chunks == decltype(NCH)::value) row_loop(NCH);
  });
  if (n_batch > 0) finish_batch();
  JM_TSTAMP(4, 0);
  asm volatile("" ::"v"(sink));                         // every counter atomic of this thread has been performed

  if (a.first_changed) {   // window tail: the last workgroup to arrive updates the images' dirty rows
    __shared__ int win_last_s;
    __syncthreads();
    if (threadIdx.x == 0)
      win_last_s = (__hip_atomic_fetch_add(a.win_done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                    (int)gridDim.x - 1);
    __syncthreads();
    if (win_last_s) {
      unsigned long long rows = 0;
      for (int n = threadIdx.x; n < a.N; n += blockDim.x) {
        const int fc = __hip_atomic_load(&a.first_changed[(size_t)n * CHG], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        a.first_changed[(size_t)n * CHG] = 0x7fffffff;
        const int d = a.dirty_lo[n];
        rows += (unsigned long long)max(0, a.row_hi - d + 1);
        a.dirty_lo[n] = min(fc, max(d, a.row_hi + 1));
      }
      if (rows) atomicAdd(a.rows_stat, rows);
      if (threadIdx.x == 0) *a.win_done = 0;
    }
  }
  JM_TSTAMP(5, 1);
  if (a.retire.enabled) finish_pass(a.retire, gridDim.x);
  JM_TSTAMP(6, 1);
}

__global__ void copy_symbols_kernel(const uint8_t* x_init, uint8_t* x, size_t total) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x)
    x[i] = x_init ? x_init[i] : 0;
}

// Clear n pieces of 16 bytes (a kernel rather than a memset so that a caller may capture it into a graph).
__global__ void zero_fill_kernel(uint4* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0, 0, 0, 0);
}

// Activations of one layer from the fragment-major buffer to a plain float [rows, width] array; slot_unit (or NULL)
// maps the storage slot of a unit to the column it is written to.  (Inspection only: no sampling path uses it.)
template <typename T>
__global__ void unpack_activations_kernel(const T* act, int k_chunks, const int* slot_unit, int rows, int width,
                                          float* out) {
  const size_t total = (size_t)rows * width;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int row = (int)(i / width), j = (int)(i % width);
    const T v = act[frag_offset<T>(row, j, k_chunks)];
    float f;
    if constexpr (std::is_same<T, float>::value) f = v; else f = bf16_to_f32(v);
    out[(size_t)row * width + (slot_unit ? slot_unit[j] : j)] = f;
  }
}

// Gumbel-max draw for categorical positions from logits held in memory:
// x[n, t] = argmax_c (z[n, t, c] + g[n, t, c]), lowest c on ties.  One wave per (row, t).
template <typename T>
__global__ __launch_bounds__(256) void gumbel_argmax_kernel(const float* __restrict__ z, int ldz,
                                                            const float* __restrict__ g, uint8_t* x, T* enc,
                                                            int enc_chunks, int* changed, const int* rows,
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
    if (xn != x[idx]) count_changed(&changed[(size_t)sample * CHG], 1);
    x[idx] = xn;
    enc[frag_offset<T>(sample, t, enc_chunks)] = Elem<T>::from_f32(((float)xn - 128.0f) * (1.0f / 128.0f));
  }
  }
  if (retire.enabled) finish_pass(retire, gridDim.x);
}

// Start of a call: x = x_init (or zeros), enc = network input of x, bookkeeping cleared.
// What the first kernel of a call also does when the whole batch is one chain: the chain's active list becomes
// its whole sample range, the per-sample counters and the call's flags are cleared (otherwise reset_rows_kernel
// and a memset do it: two more operations on the stream, each as long as a layer at batch ~100).
struct CallReset {
  int enabled;
  int* rows;
  int* rows_other;       // the chain's second list: filled with valid ids too (tiles past the active count read it)
  int* n_rows;
  int first, count, padded;
  int* changed;
  int* iters;
  int* done_ctr;
  int* flags;
  unsigned* lazy_masks;  // [3 * DERIVE_WORDS] (see DeriveArgs), or NULL
  int* frozen_words;     // [4] first position to evaluate (two, alternating by pass) and lowest changed position (two), or NULL
  // Bernoulli model started from zeros (init_state_kernel): the first hidden layer of the first pass multiplies a zero
  // input, so its activations are relu(bias) for every sample: written here (h0_out != NULL: fragment-major buffer of
  // h0_chunks chunks, h0_units units, a multiple of 4), and the first pass starts at the second hidden layer.
  const float* h0_bias;
  void* h0_out;
  int h0_chunks, h0_units;
};

__device__ __forceinline__ void call_reset(const CallReset& r) {
  if (!r.enabled) return;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < (size_t)r.padded; i += stride) {
    r.rows[i] = (int)i < r.count ? r.first + (int)i : r.first;
    r.rows_other[i] = r.first;
    if ((int)i < r.count) {
      r.changed[(size_t)(r.first + i) * CHG] = 0;
      r.iters[r.first + i] = 0;
    }
    if (r.lazy_masks && i < 3 * DERIVE_WORDS) r.lazy_masks[i] = 0u;
    if (i == 0) {
      *r.n_rows = r.count;
      *r.done_ctr = 0;
      r.done_ctr[RETIRE_CURSOR] = 0;
      *r.flags = 0;
      if (r.frozen_words) {
        r.frozen_words[0] = r.frozen_words[1] = 0;
        r.frozen_words[2] = r.frozen_words[3] = NO_CHANGE;
      }
    }
  }
}

template <typename T>
__global__ void init_state_kernel(const uint8_t* x_init, uint8_t* x, T* enc, int enc_chunks, int N, int D, int C, CallReset reset) {
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  // (zero start: the bias of this thread's first four units is requested before anything else, so that its way from
  // memory overlaps with the rest of the kernel)
  const int quads = reset.h0_out ? reset.h0_units / 4 : 1;
  const size_t items = reset.h0_out ? (size_t)N * quads : 0;
  float4 b_first = make_float4(0.f, 0.f, 0.f, 0.f);
  if (tid < items) b_first = *(const float4*)(reset.h0_bias + 4 * (int)(tid % quads));
  call_reset(reset);
  const size_t total = (size_t)N * D;
  for (size_t i = tid; i < total; i += stride) {
    const int n = (int)(i / D), t = (int)(i % D);
    const uint8_t v = x_init ? x_init[i] : 0;
    if (x) x[i] = v;
    const float e = (C == 1) ? (float)v : ((float)v - 128.0f) * (1.0f / 128.0f);
    enc[frag_offset<T>(n, t, enc_chunks)] = Elem<T>::from_f32(e);
  }
  // (what the layer kernel's epilogue computes from an all-zero product: 0 + bias, ReLU, rounded to T)
  for (size_t i = tid; i < items; i += stride) {
    const int n = (int)(i / quads), j = 4 * (int)(i % quads);
    const float4 b = i == tid ? b_first : *(const float4*)(reset.h0_bias + j);
    const float v[4] = {fmaxf(0.f + b.x, 0.f), fmaxf(0.f + b.y, 0.f), fmaxf(0.f + b.z, 0.f), fmaxf(0.f + b.w, 0.f)};
    T* dst = (T*)reset.h0_out + frag_offset<T>(n, j, reset.h0_chunks);   // (4 consecutive units are contiguous)
    if constexpr (sizeof(T) == 2)
      *(uint2*)dst = make_uint2((uint32_t)Elem<T>::from_f32(v[0]) | ((uint32_t)Elem<T>::from_f32(v[1]) << 16),
                                (uint32_t)Elem<T>::from_f32(v[2]) | ((uint32_t)Elem<T>::from_f32(v[3]) << 16));
    else
      *(uint4*)dst = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
  }
}

// Jacobi-GS (Algorithm 2), start of an iteration: every block's virtual sample starts from the previous
// iterate: xv[i * np + n] = x[n] for all blocks i, and the network input of the virtual samples is rebuilt.
template <typename T>
__global__ void jgs_begin_kernel(const uint8_t* x, uint8_t* xv, T* enc, int enc_chunks, int N, int np, int M, int D) {
  const size_t total = (size_t)M * np * D;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const int v = (int)(e / D), t = (int)(e % D);
    const int n = v % np;
    const uint8_t val = n < N ? x[(size_t)n * D + t] : 0;
    xv[e] = val;
    enc[frag_offset<T>(v, t, enc_chunks)] = Elem<T>::from_f32((float)val);
  }
}

// Algorithm 2 on the convolutional model: the N real images' symbols to all M * N virtual images (block-major:
// virtual image i * N + n is block i's copy of image n).
__global__ void jgs_conv_begin_kernel(const uint8_t* x, uint8_t* xv, int N, int M, int D) {
  const size_t per = (size_t)N * D, total = per * M;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x)
    xv[e] = x[e % per];
}

// The activations of the N real images (the first N virtual images hold them: one evaluation of the previous iterate)
// to the other blocks' copies: per layer, n16 pieces of 16 bytes per batch of N images.
__global__ void jgs_conv_broadcast_kernel(uint4* act, size_t n16, int M) {
  const size_t total = n16 * (size_t)(M - 1);
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x)
    act[n16 + e] = act[e % n16];
}

// Sub-step q of an iteration: block i's copies draw state a_i + q (none past the block's end) and need the image rows
// from the row of the state drawn before (its symbol is new) to the row of this state.
__global__ void jgs_conv_window_kernel(int* dirty_lo, int* row_hi_of, int* state_one, int N, int M, int D, int block, int q) {
  const int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= N * M) return;
  const int i = v / N, a = i * block, st = a + q;
  const bool live = st < min(a + block, D);
  state_one[v] = live ? st : -1;
  dirty_lo[v] = live ? (q > 0 ? (st - 1) / 96 : st / 96) : 0x3fffffff;
  row_hi_of[v] = live ? st / 96 : -1;
}

// End of an iteration: block i's positions are taken from its virtual sample, compared with the previous
// iterate (forward difference with tolerance 0, per sample) and stored.  One workgroup per sample.
// state[n]: 0 = still iterating, 1 = stopped.  *n_active counts the samples that go on.
__global__ void jgs_end_kernel(uint8_t* x, const uint8_t* xv, int np, int D, int block, int* iters, int* state,
                               int k, int last, int flag_unconverged, int* n_active, int* flags) {
  __shared__ int any_s;
  const int n = blockIdx.x;
  if (threadIdx.x == 0) any_s = 0;
  __syncthreads();
  int any = 0;
  for (int t = threadIdx.x; t < D; t += blockDim.x) {
    const uint8_t v = xv[((size_t)(t / block) * np + n) * D + t];
    if (v != x[(size_t)n * D + t]) {
      any = 1;
      x[(size_t)n * D + t] = v;
    }
  }
  if (any) any_s = 1;          // (benign race: every writer stores 1)
  __syncthreads();
  if (threadIdx.x == 0 && state[n] == 0) {
    iters[n] = k;
    if (!any_s || last) state[n] = 1;
    else atomicAdd(n_active, 1);
    if (any_s && last && flag_unconverged) atomicOr(flags, 1);   // still changing at a caller-given limit
  }
}

// Start of a call on a model with real states: x = x_init (or zeros) and the network input (the states
// themselves, rounded to the model's element type).
template <typename T>
__global__ void init_state_real_kernel(const float* x_init, float* x, T* enc, int enc_chunks, int N, int D, CallReset reset) {
  call_reset(reset);
  const size_t total = (size_t)N * D;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int n = (int)(i / D), t = (int)(i % D);
    const float v = x_init ? x_init[i] : 0.f;
    if (x) x[i] = v;
    enc[frag_offset<T>(n, t, enc_chunks)] = Elem<T>::from_f32(v);
  }
}

// A chain's active list becomes its whole sample range [first, first + count) again (start of a call or of
// a GS-Jacobi block).
// Entries past the count, up to the list's padded length, are read as sample ids by the tile kernels (their
// results are discarded), so they are set to a valid id of this call as well.
__global__ void reset_rows_kernel(int* rows, int* rows_other, int* n_rows, int first, int count, int padded, int* changed,
                                  int* iters, int* done_ctr, int* frozen_words) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < padded) rows[i] = i < count ? first + i : first;
  if (i < padded && rows_other) rows_other[i] = first;   // (only needed once per call: see enqueue_pass)
  if (i < count) {
    changed[(size_t)(first + i) * CHG] = 0;
    if (iters) iters[first + i] = 0;
  }
  if (i == 0) {
    *n_rows = count;
    *done_ctr = 0;
    done_ctr[RETIRE_CURSOR] = 0;
    if (frozen_words) {      // (see CallReset)
      frozen_words[0] = frozen_words[1] = 0;
      frozen_words[2] = frozen_words[3] = NO_CHANGE;
    }
  }
}

}  // namespace jm
