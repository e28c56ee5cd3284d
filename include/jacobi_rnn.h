/*
 * jacobi_rnn.h -- C ABI of the recurrent-network part of libjacobi_made.so: the backward pass of a one-layer
 * RNN solved by Jacobi iteration (Section 5.1 of the paper; backpropagation as feedforward computation,
 * Appendix A.2; network of Appendix C.1: one hidden layer of softplus units).
 *
 *     z_t = W h_{t-1} + U x_t + b,   h_t = softplus(z_t),   t = 1..T,   L = sum_t l_t(h_t)
 *     states: d_t = dL/dh_t,   d_T = g_T,   d_t = g_t + W^T (sigmoid(z_{t+1}) * d_{t+1}),   g_t = dl_t/dh_t
 *
 * Conventions (as in jacobi_made.h): every pointer is DEVICE memory, fp32, row-major, owned by the caller;
 * arrays over sequences and time are [B, T, .] with B independent sequences; calls are enqueued on `stream`
 * (a hipStream_t, NULL = default stream) and return without waiting for the device; the return value is MADE_OK
 * or a negative made_status (jacobi_made.h), made_last_error() has the message.  No call allocates memory.
 * Limits: 1 <= H <= 128; the Jacobi call additionally needs T <= rnn_jacobi_max_steps(H) (128 for H > 64,
 * 256 for H > 32, 512 otherwise): one workgroup keeps a whole sequence's iterate on chip.
 */
#ifndef JACOBI_RNN_H
#define JACOBI_RNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * rnn_forward -- the forward recurrence above, one step after the other (it produces the inputs of the backward
 * pass; the paper does not change it).
 *   W [H, H]: W[i][j] multiplies h_{t-1}[j] in unit i;  U [H, I];  b [H];  x [B, T, I];  h0 [B, H] or NULL (zeros)
 *   z, h [B, T, H]: pre-activations and hidden states (outputs)
 */
int rnn_forward(const float* W, const float* U, const float* b, const float* x, const float* h0, int32_t B, int32_t T,
                int32_t H, int32_t I, float* z, float* h, void* stream);

/*
 * rnn_backward_sequential -- the standard backward pass (Section 5.1's "feedforward" baseline): the states d_t
 * from t = T down to 1, each from the one after it.
 *   z, g [B, T, H]: pre-activations of the forward pass, direct loss gradients dl_t/dh_t;  d [B, T, H] (output)
 */
int rnn_backward_sequential(const float* W, const float* z, const float* g, int32_t B, int32_t T, int32_t H, float* d,
                            void* stream);

/*
 * rnn_backward_jacobi -- the same states by Jacobi iteration (Algorithm 1): every pass updates all T steps in
 * parallel from the previous iterate, d^k_t = g_t + W^T (sigmoid(z_{t+1}) * d^{k-1}_{t+1}).  After k passes the
 * last k steps are final (Proposition 1), so T passes give the result of rnn_backward_sequential; fewer passes give
 * "Jacobi_n" of Section 5.1, backpropagation through time truncated to n steps.
 *   d_init   : [B, T, H] initial iterate, or NULL = zeros (then d^1 = g)
 *   n_iters  : pass limit n; <= 0 or > T means T
 *   eps      : forward-difference tolerance (Section 2.2.1): a sequence stops after the first pass that moves
 *              no entry of its iterate by more than eps (max-norm over steps and units); 0 = run to the limit
 *              unless a pass changes nothing at all
 *   d        : [B, T, H] the final iterate (output)
 *   iters_out: [B] passes the sequence took, or NULL;  converged_out: [B] 1 if eps was met, 0 if the limit ended
 *              the iteration, or NULL
 * Arithmetic: the matrix product of a pass takes both operands as sums of two bf16 parts (three bf16 MFMAs per
 * product, fp32 accumulation): relative error about 2^-16 per product instead of fp32's 2^-24.
 */
int rnn_backward_jacobi(const float* W, const float* z, const float* g, const float* d_init, int32_t B, int32_t T,
                        int32_t H, int32_t n_iters, float eps, float* d, int32_t* iters_out, int32_t* converged_out,
                        void* stream);

/* rnn_jacobi_max_steps -- largest T rnn_backward_jacobi accepts for H hidden units (0 if H is out of range). */
int rnn_jacobi_max_steps(int32_t H);

/*
 * rnn_param_grads -- parameter gradients from the states (Appendix A.2: available as soon as the states are),
 * with p_t = sigmoid(z_t) * d_t, summed over all steps of all sequences:
 *   dW [H, H] = sum p_t h_{t-1}^T,   dU [H, I] = sum p_t x_t^T,   db [H] = sum p_t      (outputs, overwritten)
 *   h [B, T, H] hidden states of the forward pass;  h0 [B, H] or NULL (zeros)
 */
int rnn_param_grads(const float* z, const float* h, const float* x, const float* d, const float* h0, int32_t B, int32_t T,
                    int32_t H, int32_t I, float* dW, float* dU, float* db, void* stream);

#ifdef __cplusplus
}
#endif
#endif
