// Backward pass of a one-layer recurrent network as a Jacobi iteration (gfx950 only).
//
// Backpropagation through T time steps is feedforward computation (Appendix A.2): with d_t = dL/dh_t,
//     d_T = g_T,     d_t = g_t + W^T (sigmoid(z_{t+1}) * d_{t+1})          (softplus units, Appendix C.1),
// every state hangs on the one after it.  The standard backward pass takes the steps one by one
// (rnn_backward_seq_kernel); Jacobi iteration (Algorithm 1; "Jacobi_n" of Section 5.1 when cut after n passes)
// updates all steps at once from the previous iterate, which turns T dependent matrix-vector products into
// one [T, H] x [H, H] matrix product per pass (rnn_jacobi_kernel).
//
// Sequences are independent, so one workgroup owns one sequence for the whole call: the iterate lives in
// its LDS, the recurrent weights in registers, all passes and the forward-difference stop test run inside
// one launch.
#pragma once

#include "kernels.hpp"

namespace jm {

constexpr int RNN_WAVES = 8;
constexpr int RNN_MAX_H = 128;
constexpr int RNN_TILES_PER_WAVE = 2;

__device__ __forceinline__ float rnn_sigmoid(float z) { return 1.0f / (1.0f + expf(-z)); }
__device__ __forceinline__ float rnn_softplus(float z) { return z > 20.0f ? z : log1pf(expf(z)); }

struct RnnJacobiArgs {
  const float* W;        // [H, H], W[i][j] multiplies h_{t-1}[j] in unit i
  const float* z;        // [B, T, H] pre-activations of the forward pass
  const float* g;        // [B, T, H] direct loss gradients dl_t/dh_t
  const float* d_init;   // [B, T, H] initial iterate or NULL (zeros)
  float* d;              // [B, T, H] result
  int* iters;            // [B] or NULL
  int* converged;        // [B] or NULL: 1 = the forward difference met eps, 0 = the pass limit ended the iteration
  int B, T, H;
  int cap;               // pass limit, 1 .. T
  float eps;
};

// fp32 value = hi + lo + O(2^-17 |value|), both parts bf16 (round to nearest even; gfx950 converts in hardware)
__device__ __forceinline__ void split_bf16(float v, bf16_t& hi, bf16_t& lo) {
  const __bf16 h = (__bf16)v;
  const __bf16 l = (__bf16)(v - (float)h);
  hi = __builtin_bit_cast(bf16_t, h);
  lo = __builtin_bit_cast(bf16_t, l);
}

// One pass is D_new = G + X W with X[t] = sigmoid(z[t+1]) * D_old[t+1]: a [Tp, Hp] x [Hp, Hp] product, Tp / Hp
// = T / H rounded up to 32.  gfx950 has no fast fp32 matrix path (fp32 MFMA runs at 1/16 of the bf16 rate), so
// both operands are split into two bf16 parts and a product is three bf16 MFMAs with fp32 accumulation
// (hi*hi + hi*lo + lo*hi; the dropped lo*lo term and the split residuals are ~2^-16 of a product).
// Wave w owns column tile (32 units) w % CT for good: its two W panels (hi, lo) stay in registers, as do G,
// sigmoid(z) and the current iterate of the (at most two) 32 x 32 tiles it owns.  The MFMA takes W^T as its row
// operand, so a lane holds 4 runs of 4 consecutive units of ONE time step: inputs come in 16-byte loads and the
// new X goes back to LDS in 8-byte pieces.  X lives in LDS as two bf16 arrays [time][unit] and is updated in
// place: all waves read (MFMA phase), barrier, all waves write, barrier.
template <int CT>
__global__ __launch_bounds__(RNN_WAVES * 64) void rnn_jacobi_kernel(RnnJacobiArgs a) {
  constexpr int Hp = 32 * CT;
  constexpr int KB = Hp / 16;            // MFMA K blocks (16 wide) per tile
  constexpr int LDX = Hp + 8;            // row pitch of X in bf16 elements (16 bytes of padding)
  constexpr int TW = RNN_TILES_PER_WAVE;
  extern __shared__ __align__(16) unsigned char rnn_lds[];
  __shared__ unsigned diff_s[2];
  const int T = a.T, H = a.H;
  const int Tp = (T + 31) / 32 * 32, RT = Tp / 32;
  bf16_t* Xhi = (bf16_t*)rnn_lds;
  bf16_t* Xlo = Xhi + (size_t)Tp * LDX;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int cl = lane & 31, hh = lane >> 5;
  const int seq = blockIdx.x;
  const size_t base = (size_t)seq * T * H;
  const bool vec_ok = (H % 4 == 0) && (((uintptr_t)a.g | (uintptr_t)a.z | (uintptr_t)a.d | (uintptr_t)a.d_init) % 16 == 0);

  const int c = wave % CT, q = wave / CT, nq = (RNN_WAVES - c + CT - 1) / CT;   // waves q = 0 .. nq-1 share column tile c

  // W panels: for K block m the lane holds W[k][unit], unit = 32 c + cl, k = hh * Hp/2 + 8 m .. + 8 (any
  // assignment of K to lanes works as long as the X reads below use the same one)
  uint4 whi[KB], wlo[KB];
  {
    const int unit = c * 32 + cl;
#pragma unroll
    for (int m = 0; m < KB; ++m) {
      bf16_t h8[8], l8[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int k = hh * (Hp / 2) + 8 * m + i;
        const float w = (k < H && unit < H) ? a.W[(size_t)k * H + unit] : 0.0f;
        split_bf16(w, h8[i], l8[i]);
      }
      whi[m] = make_uint4(h8[0] | (h8[1] << 16), h8[2] | (h8[3] << 16), h8[4] | (h8[5] << 16), h8[6] | (h8[7] << 16));
      wlo[m] = make_uint4(l8[0] | (l8[1] << 16), l8[2] | (l8[3] << 16), l8[4] | (l8[5] << 16), l8[6] | (l8[7] << 16));
    }
  }

  // this wave's tiles: row (time) tiles q, q + nq.  Accumulator element e = 4 jj + i of a tile is
  // (unit = 32 c + 8 jj + 4 hh + i, time = 32 r + cl).
  float G[TW][16], S[TW][16], D[TW][16];
  bool tile_ok[TW];
  auto load4f = [&](const float* p, size_t idx, int u0, bool row_ok, float (&o)[4]) {
    if (row_ok && vec_ok && u0 + 3 < H) {
      const float4 v = *(const float4*)(p + idx);
      o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = (row_ok && u0 + i < H) ? p[idx + i] : 0.0f;
    }
  };
#pragma unroll
  for (int i = 0; i < TW; ++i) {
    const int r = q + i * nq;
    tile_ok[i] = r < RT;
    const int t = 32 * r + cl;
    const bool row_ok = tile_ok[i] && t < T;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int u0 = 32 * c + 8 * jj + 4 * hh;
      const size_t idx = base + (size_t)t * H + u0;
      float gv[4], zv[4], dv[4] = {0.f, 0.f, 0.f, 0.f};
      load4f(a.g, idx, u0, row_ok, gv);
      load4f(a.z, idx, u0, row_ok, zv);
      if (a.d_init) load4f(a.d_init, idx, u0, row_ok, dv);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        G[i][4 * jj + e] = gv[e];
        S[i][4 * jj + e] = (row_ok && u0 + e < H) ? rnn_sigmoid(zv[e]) : 0.0f;
        D[i][4 * jj + e] = dv[e];
      }
    }
  }
  // X[t-1][unit .. unit+3] = S[t] * D[t], both bf16 parts, 8 bytes each
  auto store_x = [&](int i, int jj) {
    const int t = 32 * (q + i * nq) + cl;
    if (t >= 1 && t < T) {
      bf16_t h4[4], l4[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) split_bf16(S[i][4 * jj + e] * D[i][4 * jj + e], h4[e], l4[e]);
      const int off = (t - 1) * LDX + 32 * c + 8 * jj + 4 * hh;
      *(uint2*)(Xhi + off) = make_uint2(h4[0] | (h4[1] << 16), h4[2] | (h4[3] << 16));
      *(uint2*)(Xlo + off) = make_uint2(l4[0] | (l4[1] << 16), l4[2] | (l4[3] << 16));
    }
  };

  for (int i = threadIdx.x; i < Tp * LDX / 2; i += RNN_WAVES * 64) ((unsigned*)rnn_lds)[i] = 0u, ((unsigned*)Xlo)[i] = 0u;
  if (threadIdx.x < 2) diff_s[threadIdx.x] = 0u;
  __syncthreads();
  if (a.d_init) {
#pragma unroll
    for (int i = 0; i < TW; ++i)
      if (tile_ok[i]) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) store_x(i, jj);
      }
  }
  __syncthreads();

  int k = 0, conv = 0;
  while (k < a.cap) {
    ++k;
    // ---- MFMA phase: acc^T = W^T X^T for the wave's tiles
    f32x16 acc[TW];
#pragma unroll
    for (int i = 0; i < TW; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
      if (tile_ok[i]) {
        const int xoff = (32 * (q + i * nq) + cl) * LDX + hh * (Hp / 2);
#pragma unroll
        for (int m = 0; m < KB; ++m) {
          const bf16x8 xh = __builtin_bit_cast(bf16x8, *(const uint4*)(Xhi + xoff + 8 * m));
          const bf16x8 xl = __builtin_bit_cast(bf16x8, *(const uint4*)(Xlo + xoff + 8 * m));
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, whi[m]), xl, acc[i], 0, 0, 0);
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wlo[m]), xh, acc[i], 0, 0, 0);
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, whi[m]), xh, acc[i], 0, 0, 0);
        }
      }
    }
    __syncthreads();   // every wave has read the old X
    // ---- update phase: D = G + acc, forward difference, X[t-1] = S[t] * D[t]
    float diff = 0.0f;
#pragma unroll
    for (int i = 0; i < TW; ++i) {
      if (tile_ok[i]) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float dn = G[i][4 * jj + e] + acc[i][4 * jj + e];
            const float df = fabsf(dn - D[i][4 * jj + e]);
            diff = fmaxf(diff, df == df ? df : __builtin_inff());       // (a NaN never counts as converged)
            D[i][4 * jj + e] = dn;
          }
          store_x(i, jj);
        }
      }
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) diff = fmaxf(diff, __shfl_xor(diff, s));
    if (lane == 0) atomicMax(&diff_s[k & 1], __float_as_uint(diff));   // (non-negative floats order like their bits)
    if (threadIdx.x == 0) diff_s[(k + 1) & 1] = 0u;                    // the slot of the pass after this one
    __syncthreads();
    if (__uint_as_float(diff_s[k & 1]) <= a.eps) {
      conv = 1;
      break;
    }
  }

#pragma unroll
  for (int i = 0; i < TW; ++i) {
    const int t = 32 * (q + i * nq) + cl;
    if (tile_ok[i] && t < T) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int u0 = 32 * c + 8 * jj + 4 * hh;
        float* dst = a.d + base + (size_t)t * H + u0;
        if (vec_ok && u0 + 3 < H) {
          *(float4*)dst = make_float4(D[i][4 * jj], D[i][4 * jj + 1], D[i][4 * jj + 2], D[i][4 * jj + 3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (u0 + e < H) dst[e] = D[i][4 * jj + e];
        }
      }
    }
  }
  if (threadIdx.x == 0) {
    if (a.iters) a.iters[seq] = k;
    if (a.converged) a.converged[seq] = conv;
  }
}

// out[j] = sum_k v[k] M(k, j) for one sequence and one step, shared by the forward pass (M = W^T) and the
// standard backward pass (M = W): thread (j, half) holds half of column j of M in registers and sums its half of
// K; the two halves meet through LDS.  blockDim = 2 * Hp, Hp = H rounded up to 32 (<= 128).
template <bool TRANSPOSED>
__device__ __forceinline__ void rnn_load_column(const float* W, int H, int j, int half, int kh, float (&m)[RNN_MAX_H / 2]) {
#pragma unroll
  for (int i = 0; i < RNN_MAX_H / 2; ++i) {
    const int k = half * kh + i;
    m[i] = (i < kh && k < H && j < H) ? (TRANSPOSED ? W[(size_t)j * H + k] : W[(size_t)k * H + j]) : 0.0f;
  }
}

__device__ __forceinline__ float rnn_half_dot(const float* v, int half, int kh, const float (&m)[RNN_MAX_H / 2]) {
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < RNN_MAX_H / 2; i += 4) {
    if (i < kh) {
      const float4 x = *(const float4*)(v + half * kh + i);
      s = fmaf(x.x, m[i], s);
      s = fmaf(x.y, m[i + 1], s);
      s = fmaf(x.z, m[i + 2], s);
      s = fmaf(x.w, m[i + 3], s);
    }
  }
  return s;
}

// The standard backward pass (Section 5.1's "feedforward" baseline): T dependent steps, last step first.
__global__ __launch_bounds__(2 * RNN_MAX_H) void rnn_backward_seq_kernel(const float* W, const float* z, const float* g, float* d,
                                                                         int T, int H) {
  __shared__ __align__(16) float v[RNN_MAX_H];
  __shared__ float part[RNN_MAX_H];
  const int Hp = blockDim.x / 2, kh = Hp / 2;
  const int j = threadIdx.x % Hp, half = threadIdx.x / Hp;
  const size_t base = (size_t)blockIdx.x * T * H;
  float m[RNN_MAX_H / 2];
  rnn_load_column<false>(W, H, j, half, kh, m);
  float dj = 0.0f;
  for (int t = T - 1; t >= 0; --t) {
    // inputs of this step do not depend on the recurrence: request them before the dot product
    const bool ok = j < H;
    const float gt = (ok && half == 0) ? g[base + (size_t)t * H + j] : 0.0f;
    const float st = (ok && half == 0 && t > 0) ? rnn_sigmoid(z[base + (size_t)t * H + j]) : 0.0f;
    float s = 0.0f;
    if (t < T - 1) s = rnn_half_dot(v, half, kh, m);
    if (half == 1) part[j] = s;
    __syncthreads();
    if (half == 0) {
      dj = gt + s + part[j];
      if (ok) d[base + (size_t)t * H + j] = dj;
      v[j] = st * dj;                      // the next (earlier) step reads sigmoid(z_t) * d_t
    }
    __syncthreads();
  }
}

// Forward pass: z_t = W h_{t-1} + U x_t + b, h_t = softplus(z_t), one step after the other.
__global__ __launch_bounds__(2 * RNN_MAX_H) void rnn_forward_kernel(const float* W, const float* U, const float* b, const float* x,
                                                                    const float* h0, float* z, float* h, int T, int H, int I) {
  __shared__ __align__(16) float v[RNN_MAX_H];
  __shared__ float part[RNN_MAX_H];
  const int Hp = blockDim.x / 2, kh = Hp / 2;
  const int j = threadIdx.x % Hp, half = threadIdx.x / Hp;
  const size_t base = (size_t)blockIdx.x * T * H;
  float m[RNN_MAX_H / 2];
  rnn_load_column<true>(W, H, j, half, kh, m);
  const bool ok = j < H;
  const float bj = ok ? b[j] : 0.0f;
  if (half == 0) v[j] = (ok && h0) ? h0[(size_t)blockIdx.x * H + j] : 0.0f;
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    float in = bj;
    if (half == 0 && ok)
      for (int cidx = 0; cidx < I; ++cidx) in = fmaf(U[(size_t)j * I + cidx], x[((size_t)blockIdx.x * T + t) * I + cidx], in);
    const float s = rnn_half_dot(v, half, kh, m);
    if (half == 1) part[j] = s;
    __syncthreads();
    if (half == 0) {
      const float zt = in + s + part[j];
      const float ht = rnn_softplus(zt);
      if (ok) {
        z[base + (size_t)t * H + j] = zt;
        h[base + (size_t)t * H + j] = ht;
      }
      v[j] = ok ? ht : 0.0f;
    }
    __syncthreads();
  }
}

// Parameter gradients from the states (Appendix A.2: "immediately computed" once they are known), with
// p_t = sigmoid(z_t) * d_t:   dW[i][j] = sum p_t[i] h_{t-1}[j],   dU[i][c] = sum p_t[i] x_t[c],   db[i] = sum p_t[i],
// sums over all steps of all sequences.  One workgroup per 32 x 32 tile of dW; its 8 waves split the B T rows
// and meet through LDS in a fixed order.  fp32 MFMA (K = 2 per instruction): this product runs once per call.
__global__ __launch_bounds__(RNN_WAVES * 64) void rnn_param_grads_kernel(const float* z, const float* h, const float* x, const float* d,
                                                                         const float* h0, int B, int T, int H, int I, float* dW,
                                                                         float* dU, float* db) {
  __shared__ float red[RNN_WAVES][32][33];
  const int CT = (H + 31) / 32;
  const int ti = blockIdx.x / CT, tj = blockIdx.x % CT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cl = lane & 31, hh = lane >> 5;
  const int i = ti * 32 + cl, j = tj * 32 + cl;
  const long long rows = (long long)B * T;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
  for (long long r0 = 2LL * wave; r0 < rows; r0 += 2LL * RNN_WAVES) {
    const long long r = r0 + hh;       // the MFMA contracts two rows per instruction: lane half hh takes row r0 + hh
    float p = 0.0f, prev = 0.0f;
    if (r < rows) {
      const int t = (int)(r % T);
      const long long seq = r / T;
      if (i < H) p = rnn_sigmoid(z[r * H + i]) * d[r * H + i];
      if (j < H) prev = t > 0 ? h[(r - 1) * H + j] : (h0 ? h0[seq * H + j] : 0.0f);
    }
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(p, prev, acc, 0, 0, 0);
  }
  // acc[e] = element (row = 8 (e / 4) + 4 hh + e % 4 -> unit i of the tile, col = cl -> unit j of the tile)
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][8 * (e >> 2) + 4 * hh + (e & 3)][cl] = acc[e];
  __syncthreads();
  for (int idx = threadIdx.x; idx < 32 * 32; idx += RNN_WAVES * 64) {
    const int ri = idx >> 5, cj = idx & 31;
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < RNN_WAVES; ++w) s += red[w][ri][cj];
    if (ti * 32 + ri < H && tj * 32 + cj < H) dW[(size_t)(ti * 32 + ri) * H + tj * 32 + cj] = s;
  }
  if (tj == 0) {     // db and dU for the 32 units of this tile row: thread (unit, slice) sums every 16th row
    __syncthreads();
    float* red1 = &red[0][0][0];
    const int unit = threadIdx.x & 31, slice = threadIdx.x >> 5;        // 16 slices
    const int iu = ti * 32 + unit;
    for (int cidx = -1; cidx < I; ++cidx) {
      float s = 0.0f;
      if (iu < H)
        for (long long r = slice; r < rows; r += 16) {
          const float p = rnn_sigmoid(z[r * H + iu]) * d[r * H + iu];
          s += cidx < 0 ? p : p * x[r * I + cidx];
        }
      red1[slice * 32 + unit] = s;
      __syncthreads();
      if (slice == 0 && iu < H) {
        float tot = 0.0f;
        for (int w = 0; w < 16; ++w) tot += red1[w * 32 + unit];
        if (cidx < 0) db[iu] = tot; else dU[(size_t)iu * I + cidx] = tot;
      }
      __syncthreads();
    }
  }
}

}  // namespace jm
