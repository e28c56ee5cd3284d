// Host side of the recurrent-network entry points (included by jacobi_made.hip after its error helpers).
#pragma once

#include "../../include/jacobi_rnn.h"
#include "rnn.hpp"

static int rnn_check_shape(const char* who, int B, int T, int H) {
  if (B < 0 || T < 1 || H < 1) return fail(MADE_ERR_ARG, "%s: B=%d, T=%d, H=%d out of range", who, B, T, H);
  if (H > RNN_MAX_H) return fail(MADE_ERR_ARG, "%s: H=%d, at most %d hidden units are supported", who, H, RNN_MAX_H);
  return MADE_OK;
}

extern "C" int rnn_jacobi_max_steps(int32_t H) {
  if (H < 1 || H > RNN_MAX_H) return 0;
  const int CT = (H + 31) / 32;
  return 32 * RNN_TILES_PER_WAVE * (RNN_WAVES / CT);
}

extern "C" int rnn_forward(const float* W, const float* U, const float* b, const float* x, const float* h0, int32_t B,
                           int32_t T, int32_t H, int32_t I, float* z, float* h, void* stream) {
  TRY(rnn_check_shape("rnn_forward", B, T, H));
  if (I < 1) return fail(MADE_ERR_ARG, "rnn_forward: I=%d must be >= 1", I);
  if (B == 0) return MADE_OK;   // (an empty batch has nothing to point at)
  if (!W || !U || !b || !x || !z || !h) return fail(MADE_ERR_ARG, "rnn_forward: NULL argument");
  const int Hp = round_up(H, 32);
  hipLaunchKernelGGL(rnn_forward_kernel, dim3(B), dim3(2 * Hp), 0, (hipStream_t)stream, W, U, b, x, h0, z, h, T, H, I);
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

extern "C" int rnn_backward_sequential(const float* W, const float* z, const float* g, int32_t B, int32_t T, int32_t H,
                                       float* d, void* stream) {
  TRY(rnn_check_shape("rnn_backward_sequential", B, T, H));
  if (B == 0) return MADE_OK;
  if (!W || !z || !g || !d) return fail(MADE_ERR_ARG, "rnn_backward_sequential: NULL argument");
  const int Hp = round_up(H, 32);
  hipLaunchKernelGGL(rnn_backward_seq_kernel, dim3(B), dim3(2 * Hp), 0, (hipStream_t)stream, W, z, g, d, T, H);
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

template <int CT>
static int rnn_launch_jacobi(const RnnJacobiArgs& a, size_t lds, hipStream_t s) {
  static size_t configured = 0;
  if (lds > configured) {
    HIP_TRY(hipFuncSetAttribute((const void*)rnn_jacobi_kernel<CT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    configured = lds;
  }
  hipLaunchKernelGGL(rnn_jacobi_kernel<CT>, dim3(a.B), dim3(RNN_WAVES * 64), lds, s, a);
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

extern "C" int rnn_backward_jacobi(const float* W, const float* z, const float* g, const float* d_init, int32_t B, int32_t T,
                                   int32_t H, int32_t n_iters, float eps, float* d, int32_t* iters_out,
                                   int32_t* converged_out, void* stream) {
  TRY(rnn_check_shape("rnn_backward_jacobi", B, T, H));
  if (!(eps >= 0.0f)) return fail(MADE_ERR_ARG, "rnn_backward_jacobi: eps must be >= 0");
  if (T > rnn_jacobi_max_steps(H))
    return fail(MADE_ERR_ARG, "rnn_backward_jacobi: T=%d, at most %d steps are supported with H=%d", T, rnn_jacobi_max_steps(H), H);
  if (B == 0) return MADE_OK;
  if (!W || !z || !g || !d) return fail(MADE_ERR_ARG, "rnn_backward_jacobi: NULL argument");
  RnnJacobiArgs a;
  a.W = W;
  a.z = z;
  a.g = g;
  a.d_init = d_init;
  a.d = d;
  a.iters = iters_out;
  a.converged = converged_out;
  a.B = B;
  a.T = T;
  a.H = H;
  a.cap = (n_iters <= 0 || n_iters > T) ? T : n_iters;
  a.eps = eps;
  const int CT = (H + 31) / 32, Tp = round_up(T, 32);
  const size_t lds = (size_t)2 * Tp * (32 * CT + 8) * sizeof(uint16_t);
  hipStream_t s = (hipStream_t)stream;
  switch (CT) {
    case 1: return rnn_launch_jacobi<1>(a, lds, s);
    case 2: return rnn_launch_jacobi<2>(a, lds, s);
    case 3: return rnn_launch_jacobi<3>(a, lds, s);
    default: return rnn_launch_jacobi<4>(a, lds, s);
  }
}

extern "C" int rnn_param_grads(const float* z, const float* h, const float* x, const float* d, const float* h0, int32_t B,
                               int32_t T, int32_t H, int32_t I, float* dW, float* dU, float* db, void* stream) {
  TRY(rnn_check_shape("rnn_param_grads", B, T, H));
  if (I < 1) return fail(MADE_ERR_ARG, "rnn_param_grads: I=%d must be >= 1", I);
  if (!z || !h || !x || !d || !dW || !dU || !db) return fail(MADE_ERR_ARG, "rnn_param_grads: NULL argument");
  const int CT = (H + 31) / 32;
  hipLaunchKernelGGL(rnn_param_grads_kernel, dim3(CT * CT), dim3(RNN_WAVES * 64), 0, (hipStream_t)stream, z, h, x, d, h0, B, T,
                     H, I, dW, dU, db);
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}
