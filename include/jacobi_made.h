/*
 * jacobi_made.h -- C ABI of libjacobi_made.so (MI355X / gfx950, HIP).
 *
 * Autoregressive sampling from a MADE-style masked MLP written as the feedforward
 * recurrence  s_t = h_t(u, s_{1:t-1}),  1 <= t <= T  (paper Section 2.1, Eq. 1; the
 * sampling instance is Appendix A.3: T = D positions, s_t = the t-th symbol, u = fixed
 * per-position noise) and solved either one position at a time or by the parallel
 * fixed-point iterations of Section 3: nonlinear Jacobi (Algorithm 1) and the block
 * hybrid GS-Jacobi (Algorithm 3).  With tolerance 0 all three return the same symbols
 * (Propositions 1 and 2).
 *
 * Conventions for every entry point
 *   - returns MADE_OK (0) or a negative made_status; nothing throws or aborts across the
 *     ABI; made_last_error() gives a thread-local message for the last failure.
 *   - "host" pointers are ordinary CPU memory, read during the call only.
 *   - "device" pointers are HIP device memory on the device that was current in
 *     made_init; they stay owned by the caller and are never freed or retained.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Results are
 *     ordered on `stream` like those of a kernel launch: read them from work enqueued on the
 *     same stream, or after synchronising it.  The *_sample calls with a stop test wait for
 *     the device's answer (they return once the result is final and the status is known), but
 *     a few empty launches they enqueued ahead of that answer may still be draining when they
 *     return; sequential_sample and made_forward_logits only enqueue work.
 *   - one model must not be used from two host threads at once (it owns scratch memory).
 *   - a *_sample call that waits for the device gives up after 30 s without an answer and returns MADE_ERR_HIP
 *     with its kernels possibly still queued: synchronise the device before reusing that call's buffers; the
 *     model then refuses every further call and made_free waits for the device before it releases anything.
 */
#ifndef JACOBI_MADE_H
#define JACOBI_MADE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct made_model made_model; /* opaque; owned by the library */

typedef enum made_status {
  MADE_OK = 0,
  MADE_ERR_ARG = -1,           /* NULL / out-of-range argument, inconsistent sizes        */
  MADE_ERR_NOMEM = -2,         /* host or device allocation failed                        */
  MADE_ERR_HIP = -3,           /* a HIP runtime call failed (message has the HIP error)   */
  MADE_ERR_NOT_CONVERGED = -4  /* max_iters passes ran and some sample was still changing;
                                  x_out then holds the current iterate                    */
} made_status;

enum { MADE_F32 = 0, MADE_BF16 = 1 };

typedef struct made_config {
  int32_t D;             /* number of positions (T in the paper), 2 <= D                  */
  int32_t C;             /* 1: Bernoulli positions; 2..256: C-way categorical positions    */
  int32_t n_hidden;      /* L >= 1 hidden masked layers                                   */
  const int32_t* hidden; /* host, [L] widths                                              */
  int32_t dtype;         /* MADE_F32: fp32 weights/activations; MADE_BF16: bf16 weights and
                            hidden activations (rounded to nearest even after bias+ReLU),
                            fp32 accumulation, fp32 logits                                */
  int32_t real;          /* 0: discrete positions (above).  1: real-valued positions with logistic
                            conditionals (the paper's own MADE, Appendix C.3); then C must be 2:
                            output row 2t is the mean mu_t and row 2t+1 the log-scale a_t of
                            position t, and the *_real entry points below are the ones to call */
  int32_t onehot;        /* 0: a categorical symbol enters the network as the scalar (x - 128) / 128 and W[0]
                            is [hidden[0], D].  1 (C >= 2 only): it enters as a one-hot vector, W[0] is
                            [hidden[0], D*C] with column t*C + c the weight of "x_t = c"; the first layer is
                            then b + the sum over visible positions t of column t*C + x_t (the other reading
                            of a categorical model's input; a gather instead of a matrix product)        */
} made_config;

/*
 * made_init -- build the masked network h_t is made of (the MADE the paper samples from in
 * Section 5.3.1; masks are the construction of the model it cites).
 *   degrees : host, [L] pointers; degrees[l] has hidden[l] entries in [1, D-1].
 *   W       : host, [L+1] pointers to UNMASKED row-major [out, in] fp32 matrices; layer L is
 *             the output layer with D*C rows, row t*C + c = class c of position t (0-based).
 *             With MADE_BF16 every value is converted to bf16 (nearest even).
 *   b       : host, [L+1] pointers to fp32 biases, any of them (or b itself) may be NULL = 0.
 * Masks: input position d (1-based) has degree d; a hidden unit of degree m reads units of
 * degree <= m; output rows of position t read last-layer units of degree < t.  The library
 * multiplies the masks in, reorders hidden units by degree (invisible from outside) and
 * uploads the result.  *out receives the model; release it with made_free.
 */
int made_init(const made_config* cfg, const int32_t* const* degrees, const float* const* W,
              const float* const* b, made_model** out);

/*
 * made_conv_init -- a PixelCNN-style masked convolutional network in place of the masked MLP (the paper's second
 * sampling experiment, Section 5.3.2, uses a network of this kind; states are sub-pixels in raster-scan order,
 * Section 5.3).  The image is H x 32 pixels with 3 colours; state t = (y * 32 + x) * 3 + colour, D = H * 32 * 3,
 * every state C = 256-way categorical, entering the network as (symbol - 128) / 128.
 *   W[0]          : host fp32 [F, k, k, 3]   first layer, mask type A
 *   W[1..n_conv-1]: host fp32 [F, k, k, F]   mask type B
 *   W[n_conv]     : host fp32 [3*256, F]     1 x 1 head, mask type B; rows colour*256 + class
 *   b             : [n_conv + 1] biases or NULL.  ReLU after every k x k layer.
 * Tap (ky, kx) reads the input at offset (ky - k/2, kx - k/2), zero outside the image.  Masks: taps above, or in
 * the same row to the left, are fully visible; taps below or to the right are not; at the centre tap an output
 * of group j sees inputs of group < j (type A; input colour c is group c) or <= j (type B).  The F features form
 * three groups of sizes ceil(F/3), ceil((F - s0)/2), rest; head rows of colour c are group c.
 * Supported: F in {64, 128}, k odd with 3 <= k <= 7, n_conv >= 2.  The model works with made_forward_logits, jacobi_sample,
 * gs_jacobi_sample (blocks of consecutive states; every inner pass evaluates the whole network) and
 * sequential_sample (both modes evaluate the whole network at every step: no activation cache).
 */
typedef struct made_conv_config {
  int32_t H, W;   /* image height; width (must be 32)          */
  int32_t C;      /* classes per sub-pixel (must be 256)       */
  int32_t F;      /* feature channels                          */
  int32_t k;      /* kernel size of the masked layers          */
  int32_t n_conv; /* number of k x k masked layers             */
  int32_t dtype;  /* MADE_F32 or MADE_BF16                     */
} made_conv_config;
int made_conv_init(const made_conv_config* cfg, const float* const* W, const float* const* b, made_model** out);

/* made_free -- release the model and all of its device scratch memory.  NULL is accepted. */
int made_free(made_model* m);

/*
 * made_forward_logits -- one pass over the whole network: the logits every h_t reads
 * (Section 5.3.1: one forward propagation yields all positions at once).
 *   x      : device, uint8 [N, D] symbols (Bernoulli: 0/1; categorical: 0..C-1, entering the
 *            network as the scalar (x - 128)/128 per position).
 *   logits : device, fp32 [N, D, C].
 * Asynchronous on `stream`.
 */
int made_forward_logits(made_model* m, const uint8_t* x, int32_t N, float* logits, void* stream);

/*
 * made_forward_logits_noalloc -- made_forward_logits for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * logits; the network input and the hidden activations of the pass live in a static device array of 8 MiB (one copy
 * per GPU, held until the process ends) instead of the model's workspace, and the call neither allocates, frees nor
 * waits for the device.  Only work on `stream` is enqueued (a clearing kernel, then the pass).
 *   Limit: round_up(N, 64) * (sum over the layers of their input width padded to a multiple of 64) * element size
 *   must fit the 8 MiB (D = 784 with 2 x 2000 hidden units in bf16: 832 samples per call); beyond that the call
 *   returns MADE_ERR_ARG and the message states the limit for the model.  Masked MLPs with discrete states only.
 *   All calls on one GPU share that GPU's array, whatever the model: calls that overlap in time (different streams,
 *   or graphs replayed concurrently) race on it and must be serialised by the caller.
 */
int made_forward_logits_noalloc(made_model* m, const uint8_t* x, int32_t N, float* logits, void* stream);

/*
 * made_layer_activations -- inspection aid for tests: the activations h_l = ReLU((W_l * M_l) h_{l-1} + b_l) of one
 * layer of the network of Section 5.3.1 (for the convolutional model: of one k x k layer) as the library holds
 * them, i.e. after the rounding to bf16 of a MADE_BF16 model, widened exactly to fp32.  Feeding them to a reference
 * implementation of layer l + 1 checks every layer on its own, without the compounding of rounding differences
 * over the depth of the network.
 *   x     : device uint8 [N, D] symbols; the whole network is evaluated on them first.  NULL (convolutional model
 *           only, N at most the batch of that call): nothing is evaluated, the values the most recent sampling call
 *           left in the model's per-layer buffers are returned.
 *   layer : 0 .. L-1 (masked MLP) or 0 .. n_conv-1 (convolutional model).
 *   out   : device fp32; masked MLP: [N, hidden[layer]] with the units in the caller's order; convolutional model:
 *           [N, H, 32, F].
 * Asynchronous on `stream`.  Models with real states are refused.
 */
int made_layer_activations(made_model* m, const uint8_t* x, int32_t N, int32_t layer, float* out, void* stream);

/*
 * Noise (the input u of Eq. 1, fixed for the whole call; Appendix A.3):
 *   Bernoulli  : device fp32 u[N, D] in [0, 1);  x_t = 1  iff  u_t < sigmoid(z_t)
 *   categorical: device fp32 g[N, D, C] standard Gumbel values;  x_t = argmax_c (z_tc + g_tc),
 *                lowest index on ties.
 */

/*
 * sequential_sample -- the feedforward computation itself (Section 2.1): for t = 1..D,
 * x_t = h_t(u, x_{1:t-1}).
 *   mode 0: every step runs the whole network, as the paper's baseline does (Section 5.3.1);
 *   mode 1: every step evaluates only what position t can see (hidden units of degree < t and
 *           the output rows of t) -- same result, the lean engineering baseline.
 *   x_out : device uint8 [N, D].
 */
int sequential_sample(made_model* m, const float* noise, int32_t N, int32_t mode, uint8_t* x_out,
                      void* stream);

/*
 * jacobi_sample -- Algorithm 1 with tolerance 0, each of the N samples an independent system.
 * Starting from x_init (NULL = zeros), every pass recomputes all D positions in parallel from
 * the previous iterate.  A sample stops at the first pass k that leaves it unchanged, or at
 * k = D (exact by Proposition 1); stopped samples leave the batch.
 *   max_iters : cap on passes, <= 0 or > D means D.  If the cap is below D and a sample is still
 *               changing the call returns MADE_ERR_NOT_CONVERGED.
 *   x_out     : device uint8 [N, D] (may alias x_init).
 *   iters_out : device int32 [N] or NULL; the stopping k of every sample (it counts the pass
 *               that only confirmed the fixed point).
 */
int jacobi_sample(made_model* m, const float* noise, int32_t N, const uint8_t* x_init,
                  int32_t max_iters, uint8_t* x_out, int32_t* iters_out, void* stream);

/*
 * gs_jacobi_sample -- Algorithm 3 with tolerance 0: blocks of `block` consecutive positions
 * (the last one may be short) are solved one after the other; inside block [a, b] Jacobi passes
 * update only the block's positions against the final values of earlier blocks, until the block
 * is unchanged or |block| passes ran.  Block positions start from x_init (NULL = zeros).
 *   iters_out : device int32 [N] or NULL; per sample, the sum over blocks of inner passes.
 */
int gs_jacobi_sample(made_model* m, const float* noise, int32_t N, const uint8_t* x_init,
                     int32_t block, uint8_t* x_out, int32_t* iters_out, void* stream);

/*
 * jacobi_gs_sample -- Algorithm 2 (Jacobi-GS) with tolerance 0: in every iteration all blocks of `block`
 * consecutive positions (the last one may be short) are processed "in parallel", each from the previous
 * iterate, and inside a block the positions are drawn one after the other:
 *     s_j^k = h_j(u, s^{k-1}_{1:a-1}, s^k_{a:j-1})   for j in block [a, b].
 * Per sample the iteration stops at the first k with s^k == s^{k-1}, or at k = M (number of blocks), where the
 * result is exact (Proposition 2).  One iteration costs `block` evaluations of the hidden layers on M copies
 * of the batch (every block has its own mixed input), so on a masked MLP this solver is the most expensive of
 * the family; it is here for completeness of the paper's solvers.
 *   x_init    : device uint8 [N, D] or NULL (zeros).
 *   max_iters : <= 0 or > M means M; a smaller limit makes the call return MADE_ERR_NOT_CONVERGED when a
 *               sample was still changing in the last allowed iteration (x_out then holds that iterate).
 *   iters_out : device int32 [N] or NULL; iterations per sample (including the confirming one).
 * Supported: the masked MLP with Bernoulli positions (C = 1), M * round_up(N, 32) <= 2^22; and the convolutional model
 * (blocks of consecutive sub-pixel states, e.g. 96 = one image row; Section 5.3.2 runs this solver with blocks of one
 * row): there every block works on a copy of the image of its own, M * N copies in all, whose per-layer activations
 * must fit 64 GB, and an iteration costs `block` launches of the layer stack on about one image row per copy.
 */
int jacobi_gs_sample(made_model* m, const float* noise, int32_t N, const uint8_t* x_init, int32_t block,
                     int32_t max_iters, uint8_t* x_out, int32_t* iters_out, void* stream);

/*
 * Models with real states (made_config.real = 1).  The recurrence (Eq. 1) is the inverse-CDF draw of a logistic
 * conditional (Appendix A.3): s_t = mu_t + exp(clip(a_t, -6, 3)) * l_t, where (mu_t, a_t) are the network's two
 * outputs for position t given s_{1:t-1} and l_t = log(u_t / (1 - u_t)) is the fixed noise (standard logistic
 * variates).  A state enters the network as itself (rounded to bf16 with MADE_BF16).  Algorithm 1 / 3 run with
 * the forward-difference tolerance eps of the paper (Sections 2.2, 4.2): per sample, the iteration (of a block)
 * stops at the first k where no position moved by more than eps (max-norm), or at the proven bound.  eps = 0
 * reproduces the sequential result of the same arithmetic exactly; eps > 0 trades accuracy for iterations.
 *   noise  : device fp32 [N, D] standard logistic variates
 *   x_init : device fp32 [N, D] or NULL (zeros);  x_out : device fp32 [N, D]
 *   made_forward_params: params = device fp32 [N, D, 2] = (mu, a) of every position for the given states.
 * Errors as for the discrete entry points (which refuse a model with real states, and vice versa).
 */
int made_forward_params(made_model* m, const float* x, int32_t N, float* params, void* stream);
int sequential_sample_real(made_model* m, const float* noise, int32_t N, int32_t mode, float* x_out, void* stream);
int jacobi_sample_real(made_model* m, const float* noise, int32_t N, const float* x_init, float eps,
                       int32_t max_iters, float* x_out, int32_t* iters_out, void* stream);
int gs_jacobi_sample_real(made_model* m, const float* noise, int32_t N, const float* x_init, int32_t block,
                          float eps, float* x_out, int32_t* iters_out, void* stream);

/*
 * made_last_stats -- counters of the most recent *_sample call on this model (host side):
 *   out[0] passes launched (network passes over the still-active part of the batch)
 *   out[1] sum over passes of active samples (sample-passes; the unit of algorithmic work)
 *   out[2] kernels launched
 *   out[3] host waits on the device
 *   out[4] convolutional model: image rows recomputed by the k x k layers, summed over passes and images (a pass
 *          only recomputes the rows below the first symbol that changed in the pass before); 0 otherwise
 *   out[5] passes whose stop test had no tail (MADE_OPT_LAZY_STOP_TEST: the next pass derived its list itself)
 *   out[6] jacobi_sample of a 256-class model: visible output-layer weights the call's passes multiplied per sample
 *          (a pass skips the positions below the first one its predecessor changed: MADE_OPT_FROZEN_POSITIONS);
 *          0 otherwise
 *   out[7] the same call: (sample, position) pairs its passes evaluated in the output layer (each reads 1 KB of noise)
 * n = number of int64 slots available in out (extra slots are left untouched).
 */
int made_last_stats(const made_model* m, int64_t* out, int32_t n);

/*
 * made_set_profiling -- when enabled, every masked-layer launch of the *_sample calls is bracketed by
 * HIP events on the caller's stream; made_last_profile then returns the summed duration in milliseconds
 * and the number of launches of the most recent *_sample call for: slots 0..L-1 the hidden layers, slot L
 * the output layer incl. its sampling epilogue, slot L+1 the persistent whole-call kernel (see
 * made_set_option).  n must be L+2.  Off by default (events cost time).
 */
int made_set_profiling(made_model* m, int32_t enable);
int made_last_profile(const made_model* m, double* ms, int64_t* launches, int32_t n);

/*
 * made_set_option -- execution choices that never change results.
 *   MADE_OPT_PERSISTENT (default 0): 1 = serve jacobi_sample / gs_jacobi_sample of Bernoulli models with
 *   batch <= 2048 from ONE cooperative launch that keeps a workgroup per CU resident and separates layers by
 *   a grid-wide barrier; 0 = one kernel launch per layer and pass.  Same results either way; on MI355X the
 *   per-layer launches are currently the faster of the two at batch 128, hence the default.
 *   MADE_OPT_FROZEN_POSITIONS (default 1; 0 or 1): models with 256 classes per position (fused output kernel): a pass
 *   of jacobi_sample / gs_jacobi_sample evaluates only the output positions behind the lowest position that the
 *   pass before changed in any sample still active.  The positions up to there read the inputs they read in that
 *   pass and would draw the same symbols (Proposition 1's frozen prefix, measured per pass instead of bounded by the
 *   pass count): same results, same pass counts, fewer of the output layer's weights streamed in the late passes.
 *   MADE_OPT_LAZY_STOP_TEST (default 1; 0 or 1): jacobi_sample of a Bernoulli model on at most 256 samples (per-layer
 *   launches): the sampling kernel of a pass only records which samples changed, and every workgroup of the next
 *   pass's first kernel derives that pass's list of active samples from the record -- in the memory round trip in
 *   which it would otherwise read the list -- instead of the previous pass's last workgroup compacting it in a tail
 *   of three dependent round trips.  Same results and pass counts; 0 keeps the tail.
 *   MADE_OPT_ZERO_START (default 1; 0 or 1): jacobi_sample of a Bernoulli model with x_init = NULL (one chain, per-layer
 *   launches, batches below the MADE_OPT_MID_TILE_BATCH / MADE_OPT_BIG_TILE_BATCH thresholds): the first hidden layer of
 *   the first pass multiplies an all-zero input, so the kernel that sets the call up writes its activations, ReLU(bias),
 *   itself, and the first pass starts at the second hidden layer: one launch less per call, same results bit for bit.
 *   0 = launch the layer.
 *   MADE_OPT_CALL_GRAPH (default 0; 0 or 1): calls that MADE_OPT_LAZY_STOP_TEST covers are short and bound by what the
 *   host pays per kernel launch.  With 1, the second call with the same arguments (noise, x_init, x_out and iters_out
 *   pointers, N, max_iters, flag, a stream other than the null stream; the buffers' contents may differ) records the
 *   call's launches -- state set-up plus as many passes as the call before needed -- as a HIP graph, and that call and
 *   the later ones replay it with one launch; a call that needs more passes gets them enqueued behind the graph, and the
 *   next one records again.  (The halves of the library's pass log alternate from call to call and are part of what a
 *   recording fixes: a set of arguments called again and again has two recordings, made by its third and fourth call.)
 *   Same results and pass counts.  The model keeps the 128 most recently used recordings; a
 *   change of any option or of the workspace size discards them.  The caller must not capture such a call itself.
 *   MADE_OPT_XCD_RESIDENT (default 1; 0, 1 or 2): jacobi_sample / gs_jacobi_sample of Bernoulli models in ONE launch in
 *   which every XCD (a group of compute units with an L2 of its own) iterates its own eighth of the samples through
 *   all passes, synchronising only among its own workgroups and through its own L2 -- samples are independent
 *   systems, so nothing has to cross the chip.  0 = never; 1 = where it was measured faster than one launch per layer
 *   and pass: gs_jacobi_sample up to 1024 samples (1.5-2x), jacobi_sample up to 512 samples on models whose layers are
 *   at most 1024 units wide (1.2-1.3x; on wider layers a phase of this kernel costs more than a launch); 2 = whenever
 *   the batch fits (2048 samples).  Same symbols and pass counts as the per-layer launches.  The kernel checks that its workgroups sit on the XCDs it assumes and are
 *   all resident; if not it backs out, and this and every later call on the model take the per-layer launches.
 *   MADE_OPT_FUSED_CATEGORICAL (default 1): for C = 256, draw the Gumbel-max symbols inside the output layer's
 *   kernel (logits stay in registers); 0 = write the logits to scratch memory and draw in a second kernel, as
 *   models with other C always do.
 *   MADE_OPT_CHAINS (default 1, range 1..8): the batch is cut into this many contiguous sub-batches of whole
 *   32-sample tiles, each iterated on its own internal stream (samples are independent systems), so that the
 *   chains' dependent kernel launches can overlap.  The caller's stream waits for all of them before the call
 *   returns.  With one host thread enqueuing, more chains mean proportionally more launches; at batch 128 on
 *   MI355X that costs more than the overlap gains, hence the default of a single chain.
 *   MADE_OPT_MID_TILE_BATCH (default 1536, >= 1) and MADE_OPT_BIG_TILE_BATCH (>= 1): batches (chains) of at least
 *   MID samples run the masked layers with 128 x 128 workgroup tiles staged through LDS instead of 32 x 32 tiles,
 *   those of at least BIG samples with 256 x 256 tiles (the same kernel with four times the accumulators and LDS,
 *   one workgroup per compute unit instead of two).  On the D = 784, 2 x 2000 network the 32 x 32 and 128 x 128
 *   tiles cross over near 1536 samples.  By default the hidden layers take the 256 x 256 tiles from 16384 samples on
 *   (measured 5-12 % faster there, up to 2.5x slower below 8192, where they leave compute units idle) and the
 *   sampling layer never does (slower at every batch: 0.196 against 0.175 ms at 32768); setting
 *   MADE_OPT_BIG_TILE_BATCH applies the given threshold to every layer.
 *   MADE_OPT_CONV_ROWS (default 4; 2 or 4): image rows per workgroup of the convolutional model's k x k layers.
 *   MADE_OPT_RESIDENT (default 2; 0, 1 or 2): the sample-resident kernel serves jacobi_sample / gs_jacobi_sample of
 *   Bernoulli models in ONE launch: a workgroup keeps 32 samples' iterate and hidden activations in its LDS for the
 *   whole call, streams the masked weights from L2 and runs every pass (and block) without leaving the compute
 *   unit.  It needs input plus hidden activations of 32 samples to fit 160 KB of LDS (e.g. D = 784 with 2 x 512
 *   hidden units in bf16; not 2 x 2000).  0 = never; 1 = whenever the model fits; 2 = where it pays: for
 *   gs_jacobi_sample (short passes, otherwise dominated by dependent launches: 2x and more), not for jacobi_sample
 *   (a whole-network pass streams every visible weight through one compute unit: at best even with the per-layer
 *   launches that use all of them).  Same symbols and pass counts as the per-layer path except possibly where a
 *   decision margin vanishes (see resident.hpp).
 *   MADE_OPT_PREFIX_CACHE (default 1): GS-Jacobi on the masked MLP keeps the activations of the hidden units whose
 *   inputs all lie before the current block (degree <= block start: they are final) after the block's first
 *   pass and only re-evaluates the units behind them (1); 0 re-evaluates every visible unit in every pass.  2: in
 *   addition, on batches (chains) of at least MADE_OPT_PARTIAL_SUM_BATCH samples (default 1024) and Bernoulli
 *   models, the contribution of the frozen inputs to the units that are still evaluated -- a sum that no longer
 *   changes inside the block -- is computed once, in the block's second pass, and later passes only multiply the
 *   inputs that can still change and add it (the caching argument the paper makes for its hybrid solvers, Section
 *   4.2).  The split changes the order of the fp32 sums, so a decision within rounding of its threshold may fall
 *   the other way than with 0 or 1.  Measured on the D = 784, 2 x 2000 network it does not pay at any batch up to
 *   32768 (blocks of 16: 20.1 ms against 11.5 ms with 1 and 15.6 ms with 0): a block takes about three passes, the
 *   slice of units that is still evaluated is one or two tiles wide, and its launches are bound by their fixed
 *   costs, not by the length of the sums -- hence the default of 1.
 *   MADE_OPT_RETIRE_SPLIT (default 2048, >= 1): the stop test of a pass (which samples changed, the new active
 *   list) runs inside the pass's last kernel, in the workgroup that finishes last; batches (chains) of at least
 *   this many samples run it as a kernel of its own spread over the chip (one workgroup needs ~180 us for 32768
 *   samples; the extra launch costs a few us).  Masked-MLP models only.  The active list's internal order may
 *   then differ between runs; no result depends on it.
 */
enum { MADE_OPT_PERSISTENT = 1, MADE_OPT_FUSED_CATEGORICAL = 2, MADE_OPT_CHAINS = 3, MADE_OPT_BIG_TILE_BATCH = 4,
       MADE_OPT_CONV_ROWS = 5, MADE_OPT_PREFIX_CACHE = 6, MADE_OPT_RESIDENT = 7, MADE_OPT_RETIRE_SPLIT = 8,
       MADE_OPT_MID_TILE_BATCH = 9, MADE_OPT_PARTIAL_SUM_BATCH = 10, MADE_OPT_XCD_RESIDENT = 11,
       MADE_OPT_LAZY_STOP_TEST = 12, MADE_OPT_FROZEN_POSITIONS = 13, MADE_OPT_CALL_GRAPH = 14, MADE_OPT_ZERO_START = 15 };
int made_set_option(made_model* m, int32_t option, int32_t value);

/*
 * made_layer_nnz -- multiply-accumulates one pass over one sample needs in each of the L+1 layers, counting
 * visible (mask = 1) weights only (for the convolutional model: visible weights x pixels): one pass costs
 * 2 * sum(nnz) floating-point operations, the algorithmic work of one evaluation of all h_t (Section 5.3.1).
 * n must be L+1 (L = n_conv for the convolutional model).
 */
int made_layer_nnz(const made_model* m, int64_t* nnz, int32_t n);

/* made_last_error -- message of the calling thread's most recent failure ("" if none). */
const char* made_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* JACOBI_MADE_H */
