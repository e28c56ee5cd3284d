// Sample-resident sampler of libjacobi_made.so (gfx950 only).
//
// Samples are independent systems of equations (each has its own noise), so a workgroup can own 32 of
// them for a WHOLE call: the current iterate (as the network's input), every hidden layer's
// activations, the biases and the mask tables live in its LDS, the noise of its samples in registers,
// and the only memory traffic of a pass is the stream of masked weights from L2.  All passes of
// Algorithm 1 (or all blocks and passes of Algorithm 3) run inside one launch: no grid-wide
// synchronisation, no per-layer launches, the forward-difference stop test of Section 2.2.1 is local.
// At batch ~100 the per-layer path spends most of a pass in launch gaps between dependent kernels a few
// microseconds long; here a pass costs what one CU needs to stream the visible weights once.
#pragma once

#include <limits.h>

#include "kernels.hpp"

namespace jm {

constexpr int RES_W = 8;       // waves per workgroup; each owns whole unit tiles (no split of K: one sum order)
#ifndef JM_RES_R
#define JM_RES_R 4
#endif
constexpr int RES_R = JM_RES_R;       // weight chunks a wave keeps in flight (ring of register slots)
constexpr int RES_MAXT = 4;    // output tiles a wave can own (their noise stays in registers)
constexpr int RES_ROWS = 32;   // samples per workgroup (one MFMA tile)

struct ResidentLayer {
  const void* W;
  const float* bias;
  const int* tile_kend;
  const int* cnt_lt;     // hidden layers: cnt_lt[t] = units of degree < t, t = 0..D
  int in_pad, k_chunks, n_tiles, out_dim;
  // byte offsets into the workgroup's dynamic LDS
  int lds_out;           // hidden layers: this layer's activations (fragment-major, one row group)
  int lds_bias;          // [n_tiles * 32] floats
  int lds_kend;          // [n_tiles] ints
  int lds_cnt;           // hidden layers: [D + 1] ints
};

struct ResidentArgs {
  ResidentLayer layer[PERSIST_MAX_LAYERS];
  int L;                 // hidden layers; layer[L] is the output layer
  int lds_enc;           // network input (fragment-major, one row group)
  int lds_clear;         // bytes from the start of dynamic LDS holding input and activations (zeroed at start)
  const float* noise;    // u[N, D]
  const uint8_t* x_init; // [N, D] or NULL
  uint8_t* x;            // [N, D]
  int N, D;
  int block;             // GS-Jacobi block size; >= D: plain Jacobi
  int cap;               // plain Jacobi: pass limit (<= D)
  int flag_unconverged;
  int io_aligned;        // D % 4 == 0 and noise is 16-byte aligned
  int* iters;            // [N]
  unsigned long long* ctr;    // device, zero between calls: [0] finished workgroups, [1] flags, [2] max passes, [3] sample-passes
  unsigned long long* host;   // pinned host memory: [0] flags, [1] passes, [2] sample-passes
};

// A wave walks the weight chunks of its tiles in a fixed order.  Tiles of a layer are numbered from the
// one with the longest visible K range (j = 0) down; they are dealt to the waves in a snake
// (0..7, 7..0, 0..7, ...) so that every wave gets about the same number of chunks.  The ownership never
// depends on which part of a layer a pass recomputes, so an output tile's noise can stay in its owner's
// registers for the whole call.  At the start of a pass lane (layer * 8 + m) of every wave works out the wave's
// m-th tile of that layer (chunks to read, weight address; 0 chunks = not part of this pass); the walk is then
// the set bits of one 64-bit mask in ascending order, read with scalar lane reads.  The walk of a layer is
// padded with empty items to a multiple of RES_R, so that an item's ring slot is a compile-time constant.
constexpr int RES_TPW = 8;     // tiles per wave and layer the walk can describe
enum { CUR_CHUNK = 0, CUR_PAD = 1, CUR_END = 2 };
// (an address rebuilt from integers must be typed as global memory by hand: through a generic pointer the
// loads would be flat loads, whose completion order the compiler cannot count on)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float ThreshVec __attribute__((ext_vector_type(RES_MAXT)));   // one value per owned output tile
typedef const u32x4 __attribute__((address_space(1)))* WeightPtr;
struct TileCursor {
  unsigned long long ptr;    // address of the current chunk (wave-uniform; the lane's offset is added at the load)
  int c, n;                  // current chunk / chunks of the tile; n = 0 on an empty item
  int bit, tile, state;      // bit = layer * 8 + m of the current (or last) tile
};

struct ResCtx {
  unsigned long long mask;                  // bit (layer * 8 + m) set: this wave's m-th tile of the layer is walked
  int dn, dt;                               // per lane = per bit: chunks, tile
  unsigned dlo, dhi;                        // per lane: address of the tile's weights
  int lane_off;
};


__device__ __forceinline__ int snake_j(int m, int wave) { return (m & 1) ? (m + 1) * RES_W - 1 - wave : m * RES_W + wave; }

__device__ __forceinline__ void cursor_load(TileCursor& c, const ResCtx& x, int bit) {
  c.bit = bit;
  c.n = __builtin_amdgcn_readlane(x.dn, bit);
  c.tile = __builtin_amdgcn_readlane(x.dt, bit);
  const unsigned lo = __builtin_amdgcn_readlane((int)x.dlo, bit), hi = __builtin_amdgcn_readlane((int)x.dhi, bit);
  c.ptr = ((unsigned long long)hi << 32) | lo;
  c.c = 0;
  c.state = CUR_CHUNK;
}

// The consumer of layer l starts at the wave's first tile of that layer (and has nothing to do if there is none).
__device__ __forceinline__ void cursor_enter_layer(TileCursor& c, const ResCtx& x, int layer) {
  const unsigned lm = (unsigned)(x.mask >> (8 * layer)) & 0xffu;
  c.c = 0;
  c.n = 0;
  c.bit = 8 * layer;
  c.state = CUR_END;
  if (lm != 0) cursor_load(c, x, 8 * layer + __builtin_ctz(lm));
}

// The prefetcher starts at the wave's first tile of the pass and rolls on through the layers.
__device__ __forceinline__ void cursor_enter_pass(TileCursor& c, const ResCtx& x) {
  c.c = 0;
  c.n = 0;
  c.bit = 0;
  c.state = CUR_END;
  if (x.mask != 0) cursor_load(c, x, __builtin_ctzll(x.mask));
}

// One item on.  The common case (next chunk of the same tile) is a compare and an add; everything else happens
// once per tile.  CNT_AFTER = items of the current layer walked after this step, modulo RES_R (the callers know
// it at compile time): a layer's walk only ends where it is 0.
template <int CNT_AFTER, bool ROLL>
__device__ __forceinline__ void cursor_advance(TileCursor& c, const ResCtx& x) {
  if (++c.c < c.n) {
    c.ptr += 4096;
    return;
  }
  if (c.state == CUR_END) { c.c = 0; return; }
  const unsigned long long rem = c.bit >= 63 ? 0ull : (x.mask & (~0ull << (c.bit + 1)));
  const int nb = rem ? __builtin_ctzll(rem) : 64;
  if (c.state == CUR_CHUNK && nb < 64 && (nb >> 3) == (c.bit >> 3)) { cursor_load(c, x, nb); return; }
  c.c = 0;                          // an empty item: its load re-reads the last chunk, its data is never used
  c.n = 0;
  if (CNT_AFTER != 0) { c.state = CUR_PAD; return; }
  if (!ROLL || nb == 64) { c.state = CUR_END; return; }
  cursor_load(c, x, nb);
}

// acc += W (row operand: units) x A (column operand: samples) over one K chunk
template <typename T>
__device__ __forceinline__ void mfma_chunk_w(const u32x4 (&w)[4], const uint4 (&a)[4], f32x16& acc);
template <>
__device__ __forceinline__ void mfma_chunk_w<bf16_t>(const u32x4 (&w)[4], const uint4 (&a)[4], f32x16& acc) {
#pragma unroll
  for (int s = 0; s < 4; ++s)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w[s]), __builtin_bit_cast(bf16x8, a[s]),
                                                  acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mfma_chunk_w<float>(const u32x4 (&w)[4], const uint4 (&a)[4], f32x16& acc) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w[s].x), __uint_as_float(a[s].x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w[s].y), __uint_as_float(a[s].y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w[s].z), __uint_as_float(a[s].z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(w[s].w), __uint_as_float(a[s].w), acc, 0, 0, 0);
  }
}

template <typename T> __device__ __forceinline__ void store4(T* dst, const float (&v)[4]);
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* dst, const float (&v)[4]) {
  *(uint2*)dst = make_uint2((uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16),
                            (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16));
}
template <> __device__ __forceinline__ void store4<float>(float* dst, const float (&v)[4]) {
  *(uint4*)dst = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
}
template <typename T> __device__ __forceinline__ void load4(const T* src, float (&v)[4]);
template <> __device__ __forceinline__ void load4<bf16_t>(const bf16_t* src, float (&v)[4]) {
  const uint2 u = *(const uint2*)src;
  v[0] = __uint_as_float(u.x << 16);
  v[1] = __uint_as_float(u.x & 0xffff0000u);
  v[2] = __uint_as_float(u.y << 16);
  v[3] = __uint_as_float(u.y & 0xffff0000u);
}
template <> __device__ __forceinline__ void load4<float>(const float* src, float (&v)[4]) {
  const uint4 u = *(const uint4*)src;
  v[0] = __uint_as_float(u.x);
  v[1] = __uint_as_float(u.y);
  v[2] = __uint_as_float(u.z);
  v[3] = __uint_as_float(u.w);
}

// One layer of one pass for this wave: walk its tiles of the layer, one weight chunk per step.  Each step
// first requests the chunk RES_R - 1 items ahead (the prefetcher P runs on into the following layers: weights
// do not depend on the data), then multiplies the chunk that has arrived against the activations in LDS.
// The MFMA takes the weights as its row operand, so an accumulator lane holds 16 units (4 runs of 4
// consecutive ones) of ONE sample: results go back to the fragment-major LDS layout in 8- or 16-byte pieces.
// A wave issues at most one instruction every four cycles, so the step is kept to a few dozen instructions:
// that, not memory, is what bounds a pass.
//
// Output layer: th holds, per owned tile, the logit of the noise: u < sigmoid(z) is decided as z > log(u/(1-u))
// (one compare instead of an exponential and a division per symbol; the two forms can only disagree where z is
// within rounding of the threshold, i.e. at a vanishing decision margin).
template <typename T, bool OUT>
__device__ __forceinline__ void resident_layer(const ResidentArgs& p, unsigned char* lds, const ResCtx& cx, int l,
                                               TileCursor& P, u32x4 (&ring)[RES_R][4], const ThreshVec (&th)[16],
                                               int a0, int b0, bool row_ok, int* changed_s, int* lo_s) {
  const int lane = threadIdx.x & 63, r = lane & 31, h = lane >> 5;
  const ResidentLayer& ly = p.layer[l];
  TileCursor C;
  cursor_enter_layer(C, cx, l);
  const uint4* act_in = (const uint4*)(lds + (l == 0 ? p.lds_enc : p.layer[l > 0 ? l - 1 : 0].lds_out)) + cx.lane_off;
  const float* bias = (const float*)(lds + ly.lds_bias);
  T* out = (T*)(lds + (OUT ? p.lds_enc : ly.lds_out));       // the output layer updates the network input
  const int out_chunks = p.layer[OUT ? 0 : l + 1].k_chunks;
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  while (C.state != CUR_END) {
    static_for<RES_R>([&](auto S) {
      constexpr int s = S, ps = (s + RES_R - 1) % RES_R;
      {
        WeightPtr wa = (WeightPtr)P.ptr + cx.lane_off;
#pragma unroll
        for (int q = 0; q < 4; ++q) ring[ps][q] = wa[q * 64];
      }
      cursor_advance<s, true>(P, cx);            // P stands RES_R - 1 items ahead: (s + RES_R - 1 + 1) % RES_R = s
      if (C.state == CUR_CHUNK) {
        uint4 av[4];
        const uint4* ap = act_in + C.c * 256;
#pragma unroll
        for (int q = 0; q < 4; ++q) av[q] = ap[q * 64];
        mfma_chunk_w<T>(ring[s], av, acc);
        if (C.c + 1 == C.n) {
          const int col0 = C.tile * TILE;
          if (!OUT) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              const int u0 = col0 + 8 * jj + 4 * h;
              const float4 b = *(const float4*)(bias + u0);
              const float v[4] = {fmaxf(acc[4 * jj + 0] + b.x, 0.f), fmaxf(acc[4 * jj + 1] + b.y, 0.f),
                                  fmaxf(acc[4 * jj + 2] + b.z, 0.f), fmaxf(acc[4 * jj + 3] + b.w, 0.f)};
              store4<T>(out + frag_offset<T>(r, u0, out_chunks), v);
            }
          } else {
            const int m = C.bit & 7;
            int cnt = 0, mn = INT_MAX;
            static_for<4>([&](auto JJ) {          // (compile-time indices into th: it must stay in registers)
              constexpr int jj = JJ;
              const int p0 = col0 + 8 * jj + 4 * h;
              T* e = out + frag_offset<T>(r, p0, out_chunks);
              const float4 b = *(const float4*)(bias + p0);
              const float bb[4] = {b.x, b.y, b.z, b.w};
              float old[4], nw[4];
              load4<T>(e, old);
              bool any = false;
              static_for<4>([&](auto II) {
                constexpr int i = II;
                const float t = th[4 * jj + i][m];     // (a select between the components, in registers)
                const int pos = p0 + i;
                float xn = acc[4 * jj + i] + bb[i] > t ? 1.0f : 0.0f;
                const bool live = row_ok && (unsigned)(pos - a0) < (unsigned)(b0 - a0);
                if (!live) xn = old[i];
                if (xn != old[i]) {
                  any = true;
                  cnt += 1;
                  mn = min(mn, pos);
                }
                nw[i] = xn;
              });
              if (any) store4<T>(e, nw);
            });
            if (cnt) atomicAdd(&changed_s[r], cnt);
            if (__ballot(cnt != 0) != 0) {
#pragma unroll
              for (int d = 1; d < 64; d <<= 1) mn = min(mn, __shfl_xor(mn, d));
              if (lane == 0) atomicMin(lo_s, mn);
            }
          }
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        }
      }
      cursor_advance<(s + 1) % RES_R, false>(C, cx);
    });
  }
}

template <typename T>
__global__ __launch_bounds__(RES_W * 64) void resident_sampler_kernel(ResidentArgs p) {
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ int changed_s[RES_ROWS], active_s[RES_ROWS], iters_s[RES_ROWS];
  __shared__ int plan_s[PERSIST_MAX_LAYERS][4];   // per layer of the current pass: first j, end j, K cap (elements)
  __shared__ int ltab_s[PERSIST_MAX_LAYERS][6];   // per layer: tiles, K chunks, weight address (lo, hi), offset of the K extents
  __shared__ int have_s[PERSIST_MAX_LAYERS];   // per hidden layer: units [0, have) have been computed from complete inputs
  __shared__ int lo_s, lo_pub_s, any_s, unconv_s;
  constexpr int NT = RES_W * 64;
  constexpr int KC = 2 * Elem<T>::EPL;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int N = p.N, D = p.D, L = p.L;
  const int row0 = blockIdx.x * RES_ROWS;
  const bool row_ok = row0 + r < N;

  // ---- set-up: clear input and activations (padding columns must read as zero), stage the small tables
  for (int i = threadIdx.x; i < p.lds_clear / 16; i += NT) ((uint4*)lds)[i] = make_uint4(0, 0, 0, 0);
  for (int l = 0; l <= L; ++l) {
    const ResidentLayer& ly = p.layer[l];
    float* b = (float*)(lds + ly.lds_bias);
    int* ke = (int*)(lds + ly.lds_kend);
    for (int i = threadIdx.x; i < ly.n_tiles * TILE; i += NT) b[i] = ly.bias[i];
    for (int i = threadIdx.x; i < ly.n_tiles; i += NT) ke[i] = ly.tile_kend[i];
    if (l < L) {
      int* cn = (int*)(lds + ly.lds_cnt);
      for (int i = threadIdx.x; i <= D; i += NT) cn[i] = ly.cnt_lt[i];
    }
  }
  if (threadIdx.x < RES_ROWS) {
    changed_s[threadIdx.x] = 0;
    iters_s[threadIdx.x] = 0;
  }
  if (threadIdx.x < PERSIST_MAX_LAYERS) {
    have_s[threadIdx.x] = 0;
    if ((int)threadIdx.x <= L) {
      const ResidentLayer& ly = p.layer[threadIdx.x];
      ltab_s[threadIdx.x][0] = ly.n_tiles;
      ltab_s[threadIdx.x][1] = ly.k_chunks;
      ltab_s[threadIdx.x][2] = (int)(unsigned)((unsigned long long)ly.W & 0xffffffffull);
      ltab_s[threadIdx.x][3] = (int)(unsigned)((unsigned long long)ly.W >> 32);
      ltab_s[threadIdx.x][4] = ly.lds_kend;
    }
  }
  if (threadIdx.x == 0) {
    lo_s = INT_MAX;
    unconv_s = 0;
  }
  __syncthreads();
  T* enc = (T*)(lds + p.lds_enc);
  const int enc_chunks = p.layer[0].k_chunks;
  if (p.x_init) {
    for (int i = threadIdx.x; i < RES_ROWS * D; i += NT) {
      const int rr = i / D, t = i - rr * D;
      if (row0 + rr < N)
        enc[frag_offset<T>(rr, t, enc_chunks)] = Elem<T>::from_f32((float)p.x_init[(size_t)(row0 + rr) * D + t]);
    }
  }

  // ---- the noise of the output tiles this wave owns, as thresholds on the logit (see resident_layer): lane
  // (r, h) holds sample r, positions 8*jj + 4*h + i
  const int nt_out = p.layer[L].n_tiles;
  ThreshVec nz[16];
  static_for<RES_MAXT>([&](auto I) {
    constexpr int m = I;
    const int j = snake_j(m, wave);
    const int tile = nt_out - 1 - j;
#pragma unroll
    for (int i = 0; i < 16; ++i) nz[i][m] = 2.0f;     // (no sample / no position here: the symbol stays 0)
    if (j < nt_out && row_ok) {
      const float* src = p.noise + (size_t)(row0 + r) * D;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int p0 = tile * TILE + 8 * jj + 4 * h;
        if (p.io_aligned && p0 + 3 < D) {
          const float4 v = *(const float4*)(src + p0);
          nz[4 * jj + 0][m] = v.x;
          nz[4 * jj + 1][m] = v.y;
          nz[4 * jj + 2][m] = v.z;
          nz[4 * jj + 3][m] = v.w;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (p0 + i < D) nz[4 * jj + i][m] = src[p0 + i];
        }
      }
    }
  });

  static_for<RES_MAXT * 16>([&](auto I) {     // (compile-time indices: the array must stay in registers)
    const float u = nz[I % 16][I / 16];
    // (hardware logarithms: their error, ~1e-7 absolute here, is far inside the margin the threshold form allows;
    // u = 0 gives -inf: always 1)
    nz[I % 16][I / 16] = u >= 1.0f ? __builtin_inff() : __logf(u) - __logf(1.0f - u);
  });

  ResCtx cx;
  cx.lane_off = h * 32 + r;
  u32x4 ring[RES_R][4];
  unsigned long long passes = 0;
  int lo = 0;                       // no symbol before this position changed in the pass before
  const bool gs = p.block < D;
  for (int a0 = 0; a0 < D; a0 += p.block) {
    const int b0 = min(a0 + p.block, D);          // block = 0-based positions [a0, b0)
    if (threadIdx.x < RES_ROWS) active_s[threadIdx.x] = row0 + threadIdx.x < N;
    const int cap = gs ? b0 - a0 : p.cap;
    bool go_on = true;
    for (int k = 1; k <= cap && go_on; ++k) {
      // ---- what this pass has to recompute (thread l plans layer l).  A hidden unit of degree m reads the
      // inputs before position m (0-based), output position t the last hidden layer's units of degree <= t.
      // Positions before `lo` did not change in the pass before (and `lo` never moves backwards), so units of
      // degree <= lo and the symbols up to `lo` stand; a GS-Jacobi block [a0, b0) only needs units of degree < b0.
      RES_STAMP(passes, 0);
      if ((int)threadIdx.x <= L) {
        const int l = threadIdx.x;
        const ResidentLayer& ly = p.layer[l];
        int in_limit = -1;
        if (gs) in_limit = l == 0 ? b0 - 1 : ((const int*)(lds + p.layer[l > 0 ? l - 1 : 0].lds_cnt))[b0];
        int tb, te;
        if (l < L) {
          const int* cn = (const int*)(lds + ly.lds_cnt);
          te = gs ? min(ly.n_tiles, (cn[b0] + TILE - 1) / TILE) : ly.n_tiles;
          tb = min(min(cn[min(lo + 1, D)], have_s[l]) / TILE, te);
          have_s[l] = max(have_s[l], gs ? cn[b0] : ly.out_dim);
        } else {
          te = min(ly.n_tiles, (b0 + TILE - 1) / TILE);
          tb = min(max(a0, lo) / TILE, te);
        }
        plan_s[l][0] = ly.n_tiles - te;
        plan_s[l][1] = ly.n_tiles - tb;
        plan_s[l][2] = in_limit >= 0 ? min(ly.in_pad, (in_limit + KC - 1) / KC * KC) : ly.in_pad;
      }
      lds_barrier();

      // ---- this wave's walk: lane (layer * 8 + m) describes the wave's m-th tile of that layer
      {
        const int dl = lane >> 3, dm = lane & 7;
        int dn = 0, dt = 0;
        unsigned long long dw = 0;
        if (dl <= L) {
          const int j = snake_j(dm, wave);
          if (j >= plan_s[dl][0] && j < plan_s[dl][1]) {
            dt = ltab_s[dl][0] - 1 - j;
            const int k_end = min(((const int*)(lds + ltab_s[dl][4]))[dt], plan_s[dl][2]);
            dn = max(1, (k_end + KC - 1) / KC);
            dw = (((unsigned long long)(unsigned)ltab_s[dl][3] << 32) | (unsigned)ltab_s[dl][2]) +
                 (unsigned long long)dt * (unsigned long long)ltab_s[dl][1] * 4096ull;
          }
        }
        cx.dn = dn;
        cx.dt = dt;
        cx.dlo = (unsigned)(dw & 0xffffffffull);
        cx.dhi = (unsigned)(dw >> 32);
        cx.mask = __ballot(dn > 0);
      }

      RES_STAMP(passes, 1);
      TileCursor P;
      P.ptr = (unsigned long long)p.layer[0].W;
      P.tile = 0;
      cursor_enter_pass(P, cx);
      static_for<RES_R - 1>([&](auto S) {
        WeightPtr wa = (WeightPtr)P.ptr + cx.lane_off;
#pragma unroll
        for (int q = 0; q < 4; ++q) ring[S][q] = wa[q * 64];
        cursor_advance<(S + 1) % RES_R, true>(P, cx);
      });
      RES_STAMP(passes, 2);
      for (int l = 0; l < L; ++l) {
        resident_layer<T, false>(p, lds, cx, l, P, ring, nz, a0, b0, row_ok, changed_s, &lo_s);
        RES_STAMP(passes, 3 + min(l, 1) * 2);
        lds_barrier();
        RES_STAMP(passes, 4 + min(l, 1) * 2);
      }
      resident_layer<T, true>(p, lds, cx, L, P, ring, nz, a0, b0, row_ok, changed_s, &lo_s);
      RES_STAMP(passes, 7);
      lds_barrier();

      // ---- stop test per sample (forward difference with tolerance 0): a sample whose symbols did not
      // change, or that has used up the block's passes, leaves the iteration
      bool still = false;
      if (threadIdx.x < RES_ROWS) {
        const int t = threadIdx.x;
        if (active_s[t]) {
          iters_s[t] += 1;
          const bool ch = changed_s[t] > 0;
          if (!ch || k == cap) {
            active_s[t] = 0;
            if (ch && p.flag_unconverged) unconv_s = 1;
          } else {
            still = true;
          }
        }
        changed_s[t] = 0;
      }
      if (wave == 0) {
        const unsigned long long mask = __ballot(still);
        if (threadIdx.x == 0) {
          any_s = mask != 0;
          lo_pub_s = lo_s;
          lo_s = INT_MAX;
        }
      }
      lds_barrier();
      passes += 1;
      lo = min(lo_pub_s, b0);
      go_on = any_s != 0;
    }
  }

  __syncthreads();
  // ---- results
  for (int i = threadIdx.x; i < RES_ROWS * D; i += NT) {
    const int rr = i / D, t = i - rr * D;
    if (row0 + rr < N) p.x[(size_t)(row0 + rr) * D + t] = enc[frag_offset<T>(rr, t, enc_chunks)] != (T)0 ? 1 : 0;
  }
  if (threadIdx.x < RES_ROWS && row0 + threadIdx.x < N) p.iters[row0 + threadIdx.x] = iters_s[threadIdx.x];
  if (threadIdx.x == 0) {
    unsigned long long sum = 0;
    for (int i = 0; i < RES_ROWS; ++i) sum += (unsigned long long)iters_s[i];
    // returning atomics: each has been performed before the next is issued, so the workgroup that sees the
    // full count below also sees every workgroup's contribution
    unsigned long long o = __hip_atomic_fetch_add(&p.ctr[3], sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::"v"(o));
    o = __hip_atomic_fetch_max(&p.ctr[2], passes, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::"v"(o));
    if (unconv_s) {
      o = __hip_atomic_fetch_or(&p.ctr[1], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("" ::"v"(o));
    }
    o = __hip_atomic_fetch_add(&p.ctr[0], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (o == (unsigned long long)gridDim.x - 1) {
      for (int i = 0; i < 3; ++i) {
        const unsigned long long v = __hip_atomic_load(&p.ctr[1 + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&p.host[i], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
      for (int i = 0; i < 4; ++i) __hip_atomic_store(&p.ctr[i], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace jm
