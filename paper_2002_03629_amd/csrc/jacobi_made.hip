// libjacobi_made.so: host side of the C ABI declared in include/jacobi_made.h.
//
// Host code builds the masked, degree-sorted network (made_init) and schedules passes:
//   sequential_sample  -- Eq. 1, one position per step
//   jacobi_sample      -- Algorithm 1, tolerance 0, per-sample stopping
//   gs_jacobi_sample   -- Algorithm 3, tolerance 0
// Every arithmetic step of a pass runs in the HIP kernels of kernels.hpp.
#include "../../include/jacobi_made.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <string>
#include <thread>
#include <vector>

#include "kernels.hpp"
#include "resident.hpp"
#include "onehot.hpp"

using namespace jm;

// ------------------------------------------------------------------------------------------------
// Static scratch memory of made_forward_logits_noalloc (the entry point for callers that cannot allocate).
// `scratch` is a host-side stand-in, not a device address: host code only ever uses the address that
// hipGetSymbolAddress returned for the device at hand (every device holds its own copy of the array).
// ------------------------------------------------------------------------------------------------
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)8 << 20;   // 8 MiB per device, held until the process ends
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
static void* g_scratch_ptr[NOALLOC_MAX_DEVICES] = {nullptr};
static std::mutex g_scratch_mutex;

// Device address of `scratch` on `device`, which must be the current device.  Looked up once per device.
static hipError_t scratch_address(int device, void** out) {
  *out = nullptr;
  if (device < 0 || device >= NOALLOC_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

// ------------------------------------------------------------------------------------------------
// errors
// ------------------------------------------------------------------------------------------------
static thread_local std::string g_last_error;

static int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

#define HIP_TRY(expr)                                                                               \
  do {                                                                                              \
    hipError_t e_ = (expr);                                                                         \
    if (e_ != hipSuccess)                                                                           \
      return fail(e_ == hipErrorOutOfMemory ? MADE_ERR_NOMEM : MADE_ERR_HIP, "%s failed: %s (%s:%d)", #expr, \
                  hipGetErrorString(e_), __FILE__, __LINE__);                                       \
  } while (0)

#define TRY(expr)            \
  do {                       \
    int rc_ = (expr);        \
    if (rc_ != MADE_OK) return rc_; \
  } while (0)

static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ------------------------------------------------------------------------------------------------
// model
// ------------------------------------------------------------------------------------------------
struct Layer {
  int in_dim = 0, out_dim = 0;   // real sizes
  int in_pad = 0, out_pad = 0;   // padded to multiples of 64 (zero filled)
  int k_chunks = 0;              // in_pad / (elements per 128 bytes): K chunks per row group
  int n_tiles = 0;               // out_pad / 32
  void* W = nullptr;             // device, out_pad x in_pad of T in fragment-major layout, mask applied, units sorted by degree
  float* bias = nullptr;         // device, [out_pad]
  int* tile_kend = nullptr;      // device, [n_tiles]
  std::vector<int> h_tile_kend;  // host copy
  int* cnt_lt = nullptr;         // device, hidden layers only: [D + 2] prefix lengths by degree
  int* slot_unit = nullptr;      // device, hidden layers only: [out_dim] the caller's index of the unit stored in slot j
};

// A chain is a contiguous range of the batch's samples that is iterated on its own HIP stream.  Samples are
// independent systems (each has its own noise), so chains never exchange anything; running several of them
// concurrently overlaps the dispatch latency of one chain's dependent kernels with another chain's work.
constexpr int FROZEN_WORDS = 48;     // the frozen-position words' place in a chain's counter block (see CallReset)
struct Chain {
  hipStream_t own_stream = nullptr;  // created with the chain
  hipStream_t stream = nullptr;      // the stream this call runs the chain on (the caller's when there is one chain)
  hipEvent_t done_ev = nullptr;
  int* rows[2] = {nullptr, nullptr};
  int* n_rows[2] = {nullptr, nullptr};
  int* done_ctr = nullptr;           // workgroups-finished counter of the pass's last kernel
  volatile int* h_pin = nullptr;     // pinned, device-visible: [i] = active count after this chain's i-th pass
  int* d_pin = nullptr;              // the same memory as the device addresses it
  int pin_len = 0, rows_cap = 0;
  int pin_half = 0, pin_base = 0;    // the pass log alternates between the two halves of the pinned words from call to
  unsigned calls = 0;                // call: kernels a call leaves behind (see run_chains) may still report into its half
  // per call
  int first = 0, count = 0;
  size_t block = 0;                  // index into the call's block list
  int k_enq = 0, k_conf = 0;         // passes of the current block enqueued / whose result the host has seen
  int bound_at_block_start = 0;      // the chain's size (a block restarts the list with every sample of the chain)
  int bound = 0;                     // upper limit of the active count in the current block: the chain's size, then
                                     // what the latest confirmed pass left (the list only shrinks inside a block)
  bool block_started = false, finished = false, iters_cleared = false;
  bool lazy = false;                 // this call's passes use the tail-less stop test (see DeriveArgs)
  bool frozen = false;               // this call's passes skip the output positions that cannot change (CatArgs::t_first_ptr)
  bool first_hidden_ready = false;   // the set-up kernel wrote the first hidden layer of the call's first pass (zero start)
  std::vector<char> log_first;       // per enqueued pass: was it the first of its block
};

static void free_chain(Chain& c) {
  for (int i = 0; i < 2; ++i) {
    if (c.rows[i]) (void)hipFree(c.rows[i]);
    if (c.n_rows[i]) (void)hipFree(c.n_rows[i]);
  }
  if (c.done_ctr) (void)hipFree(c.done_ctr);
  if (c.h_pin) (void)hipHostFree((void*)c.h_pin);
  if (c.done_ev) (void)hipEventDestroy(c.done_ev);
  if (c.own_stream) (void)hipStreamDestroy(c.own_stream);
  c = Chain();
}

struct Workspace {
  int N_cap = 0;
  void* enc = nullptr;               // [N_pad, D_pad] network input of the current iterate
  std::vector<void*> act;            // hidden activations, [N_pad, pad(H_l)]
  float* zbuf = nullptr;             // categorical only: logits [N, D*C]
  std::vector<float*> partial;       // GS-Jacobi partial-sum cache: per layer 0 .. L, [n_pad, out_pad] fp32 (allocated on
  int partial_cap = 0;               // first use, for partial_cap samples)
  float* zero_bias = nullptr;        // [largest out_pad] zeros: the launches that fill `partial` add no bias
  int* changed = nullptr;
  unsigned* lazy_masks = nullptr;    // [3 * DERIVE_WORDS] changed-row bits of the tail-less stop test (see DeriveArgs)
  int* iters = nullptr;
  int* call_iters = nullptr;         // where the current call counts passes per sample: the caller's iters_out, else `iters`
  bool pending = false;              // the last call returned with (empty, speculative) kernels still queued on
  hipStream_t pending_stream = nullptr;   // this stream: a call on another stream, or a reallocation, waits for them
  int* flags = nullptr;
  int n_pad = 0;
  std::vector<Chain> chains;         // independent sub-batches, each on its own stream
  hipEvent_t fork_ev = nullptr;
  unsigned* bar = nullptr;           // persistent kernel: grid barrier counter
  long long* dev_stats = nullptr;    // persistent kernel: [passes, sample-passes]
  volatile int* h_pin = nullptr;     // pinned host words: [0] flags copy, [2..5] persistent kernel's statistics
  volatile int* xcd_report = nullptr;     // pinned, device-visible: what xcd_sampler_kernel reports (8 words per XCD + flags)
  int* xcd_report_dev = nullptr;     // the same memory as the device addresses it
  unsigned xcd_calls = 0;            // calls served by xcd_sampler_kernel on this workspace
};

// Masked convolutional model (arch 1): first layer 3 -> F (type A), n_conv - 1 layers F -> F (type B), 1 x 1 head.
struct ConvNet {
  int H = 0, F = 0, k = 0, n_conv = 0, n_taps = 0;
  int wg_rows = 4;                   // image rows per workgroup of the k x k layers: made_set_option(MADE_OPT_CONV_ROWS)
  int* taps = nullptr;               // device [n_taps][2] visible taps (dy, dx), the centre tap last
  void* w0 = nullptr;                // first layer, masked [F x K0] (K = tap * 3 + colour), fragment-major
  float* b0 = nullptr;
  std::vector<void*> w;              // layers 1 .. n_conv-1: [F x n_taps*F] tap-major K, fragment-major
  std::vector<float*> bias;
  void* w_head = nullptr;            // [3*256 x F], fragment-major
  float* b_head = nullptr;
  int* head_tile_kend = nullptr;     // [3*8]
  std::vector<void*> act;            // activations of every k x k layer for the current batch capacity (they
                                     // persist between passes: see ConvWindow)
  int* win = nullptr;                // dirty_lo [win_pad], first_changed [win_pad * CHG: one word per 128-byte line and
                                     // image, the images' updates would otherwise all queue on one line], finished-workgroup counter
  int win_pad = 0;
  unsigned long long* rows_stat = nullptr;
};

// The launches of one jacobi_sample call (state set-up + `passes` passes) recorded as a HIP graph.  Kernel arguments
// are baked into the graph, so it serves exactly the call it was recorded from: same buffers, batch, pass limit, stream
// and half of the pass log.  The noise and the initial state may hold other values: every pass stops at the device-side
// list of active samples, so passes recorded behind the one that empties the list do nothing, and a call that needs
// more passes than were recorded gets them enqueued one by one behind the graph.
struct CallGraph {
  const void* noise = nullptr;
  const void* x_init = nullptr;
  void* x = nullptr;
  int32_t* iters = nullptr;
  hipStream_t stream = nullptr;
  int N = 0, cap = 0, pin_base = 0;
  bool flag_unconverged = false;
  int needed = 0;                 // passes the last call with this key needed (0: none seen yet)
  int passes = 0;                 // passes in the recorded graph
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  std::vector<char> log_first;    // the host's pass log after the recording: the same after every replay
  int64_t kernels = 0, tail_less = 0;
  uint64_t used = 0;
};
constexpr int CALL_GRAPHS_MAX = 128;

struct made_model {
  int arch = 0;                               // 0 masked MLP, 1 masked convolutional network
  bool poisoned = false;                      // a call gave up waiting for the device with its kernels still queued:
                                              // every later call is refused, made_free waits for the device first
  bool real = false;                          // MLP with real states and logistic conditionals (C = 2 rows per position)
  bool onehot = false;                        // categorical symbols enter as one-hot vectors: the first layer is a sum of
                                              // one weight row per position (layers[0].W is [D][C][out_pad], see made_init)
  float call_eps = 0.f;                       // forward-difference tolerance of the current *_real call
  ConvNet conv;
  int D = 0, C = 1, L = 0, dtype = MADE_F32, device = 0;
  std::vector<int> hidden;
  std::vector<Layer> layers;                  // L hidden + 1 output
  // cnt_lt[l][t] = number of units of hidden layer l with degree < t (t = 0..D); units are sorted by
  // degree, so these are prefix lengths
  std::vector<std::vector<int>> cnt_lt;
  Workspace ws;
  int64_t stats[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  // Jacobi-GS (Algorithm 2): symbols of the virtual samples, per-sub-step position table, per-sample state
  uint8_t* jgs_xv = nullptr;
  size_t jgs_xv_cap = 0;
  int* jgs_tab = nullptr;
  size_t jgs_tab_cap = 0;
  int* jgs_state = nullptr;                   // [N] stopped flags, then one counter of samples still iterating
  size_t jgs_state_cap = 0;
  // optional per-layer timing with HIP events on the caller's stream
  bool profiling = false;
  std::vector<hipEvent_t> ev_pool;            // pairs: [2i] before, [2i+1] after a layer launch
  std::vector<int> ev_layer;                  // layer index of pair i in the current call
  std::vector<double> prof_ms;                // [L+1] summed duration of that layer's launches, last call
  std::vector<int64_t> prof_launches;         // [L+1]
  std::vector<int64_t> nnz;                   // [L+1] visible (mask = 1) weights per layer
  int persist_grid = 0;                       // workgroups of the persistent kernel (0 = not usable)
  int prefix_cache = 1;                       // made_set_option(MADE_OPT_PREFIX_CACHE): 0 off, 1 frozen units' activations,
                                              // 2 also the frozen inputs' partial sums, for lists of partial_batch samples on
                                              // (measured slower than 1 at every batch up to 32768: not the default)
  int partial_batch = 1024;                   // made_set_option(MADE_OPT_PARTIAL_SUM_BATCH)
  int big_batch = 16384;                      // 256 x 256 tiles from here on: measured 5-12 % faster than 128 x 128 on the
                                              // hidden layers from 16384 samples on, slower below (too few workgroups) and
  bool big_output = false;                    // slower at every batch on the sampling layer (its epilogue needs a second
                                              // workgroup on the compute unit to hide behind), which therefore stays on
                                              // 128 x 128 unless made_set_option(MADE_OPT_BIG_TILE_BATCH) names a batch
  int mid_batch = 1536;                       // made_set_option(MADE_OPT_MID_TILE_BATCH): 128 x 128 tiles from here up to
                                              // big_batch; measured crossover with the 32 x 32 tiles near 1536
  int n_chains = 1;                           // made_set_option(MADE_OPT_CHAINS)
  int retire_split = 2048;                    // made_set_option(MADE_OPT_RETIRE_SPLIT); +4 % at batch 2048, +9 % at 4096 over the fused tail
  int fused_categorical = 1;                  // made_set_option(MADE_OPT_FUSED_CATEGORICAL)
  int use_persistent = 0;                     // made_set_option(MADE_OPT_PERSISTENT): 1 = the device-wide cooperative kernel
                                              // (measured slower, see header)
  int frozen_positions = 1;                   // made_set_option(MADE_OPT_FROZEN_POSITIONS): 256-class output kernel skips the
                                              // positions below the first one that changed in the pass before
  int zero_start_fill = 1;                    // made_set_option(MADE_OPT_ZERO_START): 1 = the set-up kernel writes the first hidden layer of a call started from zeros
  int call_graph = 0;                         // made_set_option(MADE_OPT_CALL_GRAPH): replay a call's launches as one HIP graph
  std::vector<CallGraph> graphs;              // at most CALL_GRAPHS_MAX of them, least recently used goes first
  uint64_t graph_clock = 0;
  int lazy_retire = 1;                        // made_set_option(MADE_OPT_LAZY_STOP_TEST): 1 = Jacobi on lists of up to 256 samples
                                              // derives a pass's list in its first kernel instead of in the previous one's tail
  int use_xcd = 1;                            // made_set_option(MADE_OPT_XCD_RESIDENT): 0 never, 1 where it pays, 2 whenever possible
  int xcd_grid = 0;                           // workgroups of xcd_sampler_kernel (0 = not usable on this device / model)
  // sample-resident kernel (resident_sampler_kernel): LDS layout, 0 bytes = this model does not fit
  int use_resident = 2;                       // made_set_option(MADE_OPT_RESIDENT): 0 never, 1 whenever it fits, 2 where it pays
  int res_lds_bytes = 0, res_lds_enc = 0, res_lds_clear = 0;
  std::vector<int> res_lds_out, res_lds_bias, res_lds_kend, res_lds_cnt;
  unsigned long long* res_ctr = nullptr;      // device, 4 words, zero between calls
  volatile unsigned long long* res_host = nullptr;   // pinned, 3 words
};


static uint16_t host_f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static size_t elem_size(const made_model* m) { return m->dtype == MADE_BF16 ? 2 : 4; }
static int chunk_elems(const made_model* m) { return m->dtype == MADE_BF16 ? 64 : 32; }

// Recorded calls point into the workspace and depend on the options: gone with either.  (A graph may still be
// executing: wait for the device first.)
static void drop_call_graphs(made_model* m) {
  if (m->graphs.empty()) return;
  (void)hipDeviceSynchronize();
  for (CallGraph& g : m->graphs) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (g.graph) (void)hipGraphDestroy(g.graph);
  }
  m->graphs.clear();
}

static void free_workspace(Workspace& w) {
  if (w.enc) (void)hipFree(w.enc);
  for (void* p : w.act)
    if (p) (void)hipFree(p);
  if (w.zbuf) (void)hipFree(w.zbuf);
  for (float* p : w.partial)
    if (p) (void)hipFree(p);
  if (w.zero_bias) (void)hipFree(w.zero_bias);
  for (Chain& c : w.chains) free_chain(c);
  w.chains.clear();
  if (w.fork_ev) (void)hipEventDestroy(w.fork_ev);
  if (w.bar) (void)hipFree(w.bar);
  if (w.dev_stats) (void)hipFree(w.dev_stats);
  if (w.changed) (void)hipFree(w.changed);
  if (w.lazy_masks) (void)hipFree(w.lazy_masks);
  if (w.iters) (void)hipFree(w.iters);
  if (w.flags) (void)hipFree(w.flags);
  if (w.h_pin) (void)hipHostFree((void*)w.h_pin);
  if (w.xcd_report) (void)hipHostFree((void*)w.xcd_report);
  w = Workspace();
}

// Work a previous call left queued only touches the model's scratch memory.  It is ordered before anything a new
// call enqueues on the same stream; a call on a different stream has to wait for it.
static int settle(made_model* m, hipStream_t s) {
  Workspace& w = m->ws;
  if (w.pending && w.pending_stream != s) HIP_TRY(hipStreamSynchronize(w.pending_stream));
  if (w.pending && w.pending_stream != s) w.pending = false;
  return MADE_OK;
}

static int ensure_workspace(made_model* m, int N, bool need_z) {
  Workspace& w = m->ws;
  if (w.pending && (N > w.N_cap || (need_z && m->C > 1 && !w.zbuf))) {   // about to free memory queued kernels may use
    HIP_TRY(hipDeviceSynchronize());
    w.pending = false;
  }
  if (m->arch == 1) {
    if (N <= w.N_cap) return MADE_OK;
    const int cap = std::max(N, w.N_cap);
    drop_call_graphs(m);
    free_workspace(w);
    ConvNet& cv = m->conv;
    for (void* p : cv.act)
      if (p) (void)hipFree(p);
    cv.act.assign(cv.n_conv, nullptr);
    for (int i = 0; i < cv.n_conv; ++i) {
      const size_t bytes = (size_t)cap * cv.H * 32 * cv.F * elem_size(m);
      HIP_TRY(hipMalloc(&cv.act[i], bytes));
      HIP_TRY(hipMemset(cv.act[i], 0, bytes));
    }
    if (cv.win) (void)hipFree(cv.win);
    cv.win = nullptr;
    cv.win_pad = round_up(cap, 2 * TILE);
    HIP_TRY(hipMalloc((void**)&cv.win, ((size_t)cv.win_pad * (1 + CHG) + 1) * sizeof(int)));
    if (!cv.rows_stat) HIP_TRY(hipMalloc((void**)&cv.rows_stat, sizeof(unsigned long long)));
    const int n_pad = round_up(cap, 2 * TILE);
    HIP_TRY(hipEventCreateWithFlags(&w.fork_ev, hipEventDisableTiming));
    HIP_TRY(hipMalloc((void**)&w.changed, (size_t)2 * n_pad * CHG * sizeof(int)));   // one counter per 128-byte line
    w.n_pad = n_pad;
    HIP_TRY(hipMalloc((void**)&w.iters, (size_t)n_pad * sizeof(int)));
    HIP_TRY(hipMalloc((void**)&w.flags, sizeof(int)));
    HIP_TRY(hipHostMalloc((void**)&w.h_pin, 8 * sizeof(int), hipHostMallocDefault));
    w.N_cap = cap;
    return MADE_OK;
  }
  need_z = need_z && m->C > 1;
  if (N <= w.N_cap && (!need_z || w.zbuf)) return MADE_OK;
  const int cap = std::max(N, w.N_cap);
  const bool had_z = w.zbuf != nullptr;
  drop_call_graphs(m);
  free_workspace(w);
  const int n_pad = round_up(cap, 2 * TILE);   // the 64-sample kernels read list entries of a whole tile pair
  const size_t es = elem_size(m);
  const size_t enc_bytes = (size_t)n_pad * m->layers[0].in_pad * es;
  HIP_TRY(hipMalloc(&w.enc, enc_bytes));
  HIP_TRY(hipMemset(w.enc, 0, enc_bytes));
  w.act.assign(m->L, nullptr);
  for (int l = 0; l < m->L; ++l) {
    const size_t bytes = (size_t)n_pad * m->layers[l + 1].in_pad * es;
    HIP_TRY(hipMalloc(&w.act[l], bytes));
    HIP_TRY(hipMemset(w.act[l], 0, bytes));
  }
  if ((need_z || had_z) && m->C > 1) {
    HIP_TRY(hipMalloc((void**)&w.zbuf, (size_t)cap * m->D * m->C * sizeof(float)));
  }
  HIP_TRY(hipEventCreateWithFlags(&w.fork_ev, hipEventDisableTiming));
  HIP_TRY(hipMalloc((void**)&w.changed, (size_t)2 * n_pad * CHG * sizeof(int)));   // one counter per 128-byte line
  HIP_TRY(hipMalloc((void**)&w.lazy_masks, (size_t)64 * sizeof(unsigned)));
  HIP_TRY(hipMemset(w.lazy_masks, 0, (size_t)64 * sizeof(unsigned)));
  w.n_pad = n_pad;
  // (xcd_sampler_kernel: per XCD a flag array for its barrier and a counter for the registration of its workgroups,
  // and the word in which it keeps counting its barriers from call to call)
  HIP_TRY(hipMalloc((void**)&w.bar, (size_t)(2 * XCDS * XCD_LINE + XCDS * 32) * sizeof(unsigned)));
  HIP_TRY(hipMemset(w.bar, 0, (size_t)(2 * XCDS * XCD_LINE + XCDS * 32) * sizeof(unsigned)));
  HIP_TRY(hipHostMalloc((void**)&w.xcd_report, (size_t)(8 * XCDS + 8) * sizeof(int), hipHostMallocMapped));
  HIP_TRY(hipHostGetDevicePointer((void**)&w.xcd_report_dev, (void*)w.xcd_report, 0));
  for (int i = 0; i < 8 * XCDS + 8; ++i) w.xcd_report[i] = 0;
  w.xcd_calls = 0;
  HIP_TRY(hipMalloc((void**)&w.dev_stats, (size_t)2 * XCDS * sizeof(long long)));
  HIP_TRY(hipMalloc((void**)&w.iters, (size_t)n_pad * sizeof(int)));
  HIP_TRY(hipMalloc((void**)&w.flags, sizeof(int)));
  HIP_TRY(hipMemset(w.flags, 0, sizeof(int)));
  HIP_TRY(hipHostMalloc((void**)&w.h_pin, (8 + 4 * XCDS) * sizeof(int), hipHostMallocDefault));
  w.N_cap = cap;
  return MADE_OK;
}

// Chain i of n_chains with room for rows_cap samples and a pass log of pin_len entries.
static int ensure_chain(made_model* m, size_t i, int rows_cap, int pin_len) {
  Workspace& w = m->ws;
  if (w.chains.size() <= i) w.chains.resize(i + 1);
  Chain& c = w.chains[i];
  if (c.own_stream && c.rows_cap >= rows_cap && c.pin_len >= pin_len) return MADE_OK;
  if (w.pending) {
    HIP_TRY(hipDeviceSynchronize());
    w.pending = false;
  }
  drop_call_graphs(m);
  free_chain(c);
  rows_cap = round_up(rows_cap, 2 * TILE);
  HIP_TRY(hipStreamCreateWithFlags(&c.own_stream, hipStreamNonBlocking));
  HIP_TRY(hipEventCreateWithFlags(&c.done_ev, hipEventDisableTiming));
  for (int b = 0; b < 2; ++b) {
    HIP_TRY(hipMalloc((void**)&c.rows[b], (size_t)rows_cap * sizeof(int)));
    HIP_TRY(hipMemset(c.rows[b], 0, (size_t)rows_cap * sizeof(int)));   // kernels may read past the active count
    HIP_TRY(hipMalloc((void**)&c.n_rows[b], sizeof(int)));
  }
  // (the retire kernel's list cursor lives RETIRE_CURSOR words behind the counter)
  HIP_TRY(hipMalloc((void**)&c.done_ctr, (size_t)2 * RETIRE_CURSOR * sizeof(int)));
  HIP_TRY(hipMemset(c.done_ctr, 0, (size_t)2 * RETIRE_CURSOR * sizeof(int)));
  // (second half: per pass, the first position the NEXT pass evaluates -- see CatArgs::t_first_ptr)
  HIP_TRY(hipHostMalloc((void**)&c.h_pin, (size_t)2 * pin_len * sizeof(int), hipHostMallocMapped));
  HIP_TRY(hipHostGetDevicePointer((void**)&c.d_pin, (void*)c.h_pin, 0));
  c.rows_cap = rows_cap;
  c.pin_len = pin_len;
  return MADE_OK;
}

extern "C" int made_free(made_model* m) {
  if (!m) return MADE_OK;
  if (m->ws.pending) (void)hipDeviceSynchronize();
  drop_call_graphs(m);
  for (Layer& l : m->layers) {
    if (l.W) (void)hipFree(l.W);
    if (l.bias) (void)hipFree(l.bias);
    if (l.tile_kend) (void)hipFree(l.tile_kend);
    if (l.cnt_lt) (void)hipFree(l.cnt_lt);
    if (l.slot_unit) (void)hipFree(l.slot_unit);
  }
  free_workspace(m->ws);
  if (m->jgs_xv) (void)hipFree(m->jgs_xv);
  if (m->jgs_tab) (void)hipFree(m->jgs_tab);
  if (m->jgs_state) (void)hipFree(m->jgs_state);
  {
    ConvNet& cv = m->conv;
    void* ptrs[] = {cv.taps, cv.w0, cv.b0, cv.w_head, cv.b_head, cv.head_tile_kend, cv.win, cv.rows_stat};
    for (void* p : ptrs)
      if (p) (void)hipFree(p);
    for (void* p : cv.w)
      if (p) (void)hipFree(p);
    for (float* p : cv.bias)
      if (p) (void)hipFree(p);
    for (void* p : cv.act)
      if (p) (void)hipFree(p);
  }
  if (m->res_ctr) (void)hipFree(m->res_ctr);
  if (m->res_host) (void)hipHostFree((void*)m->res_host);
  for (hipEvent_t e : m->ev_pool) (void)hipEventDestroy(e);
  delete m;
  return MADE_OK;
}

extern "C" const char* made_last_error(void) { return g_last_error.c_str(); }

extern "C" int made_last_stats(const made_model* m, int64_t* out, int32_t n) {
  if (!m || !out || n < 0) return fail(MADE_ERR_ARG, "made_last_stats: NULL argument");
  for (int i = 0; i < n && i < 8; ++i) out[i] = m->stats[i];
  return MADE_OK;
}

extern "C" int made_set_profiling(made_model* m, int32_t enable) {
  if (!m) return fail(MADE_ERR_ARG, "made_set_profiling: model is NULL");
  m->profiling = enable != 0;
  return MADE_OK;
}

extern "C" int made_last_profile(const made_model* m, double* ms, int64_t* launches, int32_t n) {
  if (!m || !ms || !launches) return fail(MADE_ERR_ARG, "made_last_profile: NULL argument");
  if (n != m->L + 2) return fail(MADE_ERR_ARG, "made_last_profile: n=%d, expected L+2=%d", n, m->L + 2);
  for (int i = 0; i < n; ++i) { ms[i] = m->prof_ms[i]; launches[i] = m->prof_launches[i]; }
  return MADE_OK;
}

extern "C" int made_set_option(made_model* m, int32_t option, int32_t value) {
  if (!m) return fail(MADE_ERR_ARG, "made_set_option: model is NULL");
  drop_call_graphs(m);   // (recorded calls were shaped by the options in force)
  if (option == MADE_OPT_ZERO_START) {
    if (value != 0 && value != 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_ZERO_START=%d must be 0 or 1", value);
    m->zero_start_fill = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_CALL_GRAPH) {
    if (value != 0 && value != 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_CALL_GRAPH=%d must be 0 or 1", value);
    m->call_graph = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_PERSISTENT) {
    m->use_persistent = value != 0;
    return MADE_OK;
  }
  if (option == MADE_OPT_FROZEN_POSITIONS) {
    if (value != 0 && value != 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_FROZEN_POSITIONS=%d must be 0 or 1", value);
    m->frozen_positions = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_LAZY_STOP_TEST) {
    if (value != 0 && value != 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_LAZY_STOP_TEST=%d must be 0 or 1", value);
    m->lazy_retire = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_XCD_RESIDENT) {
    if (value < 0 || value > 2) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_XCD_RESIDENT=%d outside [0, 2]", value);
    m->use_xcd = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_FUSED_CATEGORICAL) {
    m->fused_categorical = value != 0;
    return MADE_OK;
  }
  if (option == MADE_OPT_RESIDENT) {
    if (value < 0 || value > 2) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_RESIDENT=%d outside [0, 2]", value);
    m->use_resident = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_PREFIX_CACHE) {
    if (value < 0 || value > 2) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_PREFIX_CACHE=%d outside [0, 2]", value);
    m->prefix_cache = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_PARTIAL_SUM_BATCH) {
    if (value < 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_PARTIAL_SUM_BATCH=%d must be >= 1", value);
    m->partial_batch = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_CONV_ROWS) {
    if (value != 2 && value != 4) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_CONV_ROWS=%d, supported: 2, 4", value);
    m->conv.wg_rows = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_BIG_TILE_BATCH) {
    if (value < 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_BIG_TILE_BATCH=%d must be >= 1", value);
    m->big_batch = value;
    m->big_output = true;
    return MADE_OK;
  }
  if (option == MADE_OPT_MID_TILE_BATCH) {
    if (value < 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_MID_TILE_BATCH=%d must be >= 1", value);
    m->mid_batch = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_RETIRE_SPLIT) {
    if (value < 1) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_RETIRE_SPLIT=%d must be >= 1", value);
    m->retire_split = value;
    return MADE_OK;
  }
  if (option == MADE_OPT_CHAINS) {
    if (value < 1 || value > 8) return fail(MADE_ERR_ARG, "made_set_option: MADE_OPT_CHAINS=%d outside [1, 8]", value);
    m->n_chains = value;
    return MADE_OK;
  }
  return fail(MADE_ERR_ARG, "made_set_option: unknown option %d", option);
}

extern "C" int made_layer_nnz(const made_model* m, int64_t* nnz, int32_t n) {
  if (!m || !nnz) return fail(MADE_ERR_ARG, "made_layer_nnz: NULL argument");
  if (n != m->L + 1) return fail(MADE_ERR_ARG, "made_layer_nnz: n=%d, the model has %d layers", n, m->L + 1);
  for (int i = 0; i < n; ++i) nnz[i] = m->nnz[i];
  return MADE_OK;
}

static int validate_config(const made_config* cfg, const int32_t* const* degrees, const float* const* W) {
  if (!cfg || !degrees || !W) return fail(MADE_ERR_ARG, "made_init: NULL argument");
  if (cfg->D < 2 || cfg->D > (1 << 20)) return fail(MADE_ERR_ARG, "made_init: D=%d out of range [2, 2^20]", cfg->D);
  if (cfg->C < 1 || cfg->C > 256) return fail(MADE_ERR_ARG, "made_init: C=%d out of range [1, 256]", cfg->C);
  if (cfg->n_hidden < 1 || cfg->n_hidden > 64 || !cfg->hidden)
    return fail(MADE_ERR_ARG, "made_init: n_hidden=%d out of range [1, 64] or hidden NULL", cfg->n_hidden);
  if (cfg->dtype != MADE_F32 && cfg->dtype != MADE_BF16) return fail(MADE_ERR_ARG, "made_init: unknown dtype %d", cfg->dtype);
  if ((int64_t)cfg->D * cfg->C > (int64_t)1 << 28) return fail(MADE_ERR_ARG, "made_init: D*C too large");
  if (cfg->real != 0 && cfg->real != 1) return fail(MADE_ERR_ARG, "made_init: real=%d must be 0 or 1", cfg->real);
  if (cfg->real && cfg->C != 2)
    return fail(MADE_ERR_ARG, "made_init: a model with real states has C = 2 output rows per position, not %d", cfg->C);
  if (cfg->onehot != 0 && cfg->onehot != 1) return fail(MADE_ERR_ARG, "made_init: onehot=%d must be 0 or 1", cfg->onehot);
  if (cfg->onehot && (cfg->C < 2 || cfg->real))
    return fail(MADE_ERR_ARG, "made_init: one-hot input is for categorical positions (C >= 2, discrete states)");
  for (int l = 0; l < cfg->n_hidden; ++l) {
    if (cfg->hidden[l] < 1 || cfg->hidden[l] > (1 << 20))
      return fail(MADE_ERR_ARG, "made_init: hidden[%d]=%d out of range", l, cfg->hidden[l]);
    if (!degrees[l] || !W[l]) return fail(MADE_ERR_ARG, "made_init: degrees[%d] or W[%d] is NULL", l, l);
    for (int k = 0; k < cfg->hidden[l]; ++k)
      if (degrees[l][k] < 1 || degrees[l][k] > cfg->D - 1)
        return fail(MADE_ERR_ARG, "made_init: degrees[%d][%d]=%d outside [1, D-1]", l, k, degrees[l][k]);
  }
  if (!W[cfg->n_hidden]) return fail(MADE_ERR_ARG, "made_init: W[%d] (output layer) is NULL", cfg->n_hidden);
  return MADE_OK;
}

extern "C" int made_init(const made_config* cfg, const int32_t* const* degrees, const float* const* W,
                         const float* const* b, made_model** out) {
  if (!out) return fail(MADE_ERR_ARG, "made_init: out is NULL");
  *out = nullptr;
  TRY(validate_config(cfg, degrees, W));
  made_model* m = new (std::nothrow) made_model();
  if (!m) return fail(MADE_ERR_NOMEM, "made_init: host allocation failed");
  m->D = cfg->D;
  m->C = cfg->C;
  m->real = cfg->real != 0;
  m->onehot = cfg->onehot != 0;
  m->L = cfg->n_hidden;
  m->dtype = cfg->dtype;
  m->hidden.assign(cfg->hidden, cfg->hidden + cfg->n_hidden);
  hipError_t e = hipGetDevice(&m->device);
  if (e != hipSuccess) {
    delete m;
    return fail(MADE_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  }

  {   // the static scratch array's address on this device (see made_forward_logits_noalloc)
    void* sp = nullptr;
    e = scratch_address(m->device, &sp);
    if (e != hipSuccess) {
      delete m;
      return fail(MADE_ERR_HIP, "made_init: hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    }
  }

  const int L = m->L, D = m->D, C = m->C;
  // in_deg[i]: degree of input i of the current layer, in its storage order; perm_prev maps storage
  // order -> caller's column index.
  std::vector<int> in_deg(D), perm_prev(D);
  for (int d = 0; d < D; ++d) { in_deg[d] = d + 1; perm_prev[d] = d; }
  m->layers.resize(L + 1);
  m->cnt_lt.resize(L);

  int rc = MADE_OK;
  try {
    for (int l = 0; l <= L && rc == MADE_OK; ++l) {
      Layer& ly = m->layers[l];
      const bool is_out = (l == L);
      ly.in_dim = (int)in_deg.size();
      ly.out_dim = is_out ? D * C : m->hidden[l];
      ly.in_pad = round_up(ly.in_dim, 64);
      ly.k_chunks = ly.in_pad / chunk_elems(m);
      ly.out_pad = round_up(ly.out_dim, 64);
      ly.n_tiles = ly.out_pad / TILE;

      // storage order of the output units and their degree threshold
      std::vector<int> perm(ly.out_dim), out_deg(ly.out_dim);
      if (is_out) {
        for (int j = 0; j < ly.out_dim; ++j) { perm[j] = j; out_deg[j] = j / C + 1; }  // position t (1-based)
      } else {
        std::iota(perm.begin(), perm.end(), 0);
        const int32_t* dg = degrees[l];
        std::stable_sort(perm.begin(), perm.end(), [dg](int a2, int b2) { return dg[a2] < dg[b2]; });
        for (int j = 0; j < ly.out_dim; ++j) out_deg[j] = dg[perm[j]];
        std::vector<int>& cl = m->cnt_lt[l];
        cl.assign(D + 2, 0);
        for (int t = 0; t <= D + 1; ++t)
          cl[t] = (int)(std::lower_bound(out_deg.begin(), out_deg.end(), t) - out_deg.begin());
      }
      // visible prefix per output unit: inputs are sorted by degree, so "degree <= m" (hidden) or
      // "degree < t" (output) is a prefix of the K axis
      std::vector<int> klen(ly.out_dim);
      for (int j = 0; j < ly.out_dim; ++j) {
        if (is_out)
          klen[j] = (int)(std::lower_bound(in_deg.begin(), in_deg.end(), out_deg[j]) - in_deg.begin());
        else
          klen[j] = (int)(std::upper_bound(in_deg.begin(), in_deg.end(), out_deg[j]) - in_deg.begin());
      }
      m->nnz.push_back(std::accumulate(klen.begin(), klen.end(), (int64_t)0));
      const int kc = chunk_elems(m);
      ly.h_tile_kend.assign(ly.n_tiles, 0);
      for (int j = 0; j < ly.out_dim; ++j) {
        int& te = ly.h_tile_kend[j / TILE];
        te = std::max(te, round_up(klen[j], kc));
      }

      const bool gather = (l == 0 && m->onehot);
      if (gather) {
        // every visible position contributes exactly one weight per unit and sample
        m->nnz.back() = 0;
        for (int j = 0; j < ly.out_dim; ++j) m->nnz.back() += out_deg[j];
      }
      const size_t n_w = gather ? (size_t)D * C * ly.out_pad : (size_t)ly.out_pad * ly.in_pad;
      const size_t es = elem_size(m);
      std::vector<uint8_t> host(n_w * es, 0);
      const float* Wl = W[l];
      // One-hot first layer: the caller's W[0] is [hidden[0], D*C] (column t*C + c = symbol c at position t).  It is
      // stored as [D][C][out_pad]: the row of (t, c) holds that column for all units in degree order, zero for
      // the units that may not see position t (degree <= t, 0-based t: a prefix of the row).
      auto fill_gather = [&](int t0, int t1) {
        for (int t = t0; t < t1; ++t)
          for (int c2 = 0; c2 < C; ++c2) {
            const size_t row = ((size_t)t * C + c2) * ly.out_pad;
            for (int j = 0; j < ly.out_dim; ++j) {
              if (out_deg[j] < t + 1) continue;
              const float v = Wl[(size_t)perm[j] * ((size_t)D * C) + (size_t)t * C + c2];
              if (m->dtype == MADE_BF16) ((uint16_t*)host.data())[row + j] = host_f32_to_bf16(v);
              else ((float*)host.data())[row + j] = v;
            }
          }
      };
      // mask, permute, convert and lay out in fragment-major order; rows are independent, so large layers
      // (the 2 GiB output layer of a 256-class model) are filled by several host threads
      auto fill_rows = [&](int j0, int j1) {
        for (int j = j0; j < j1; ++j) {
          const float* src = Wl + (size_t)perm[j] * ly.in_dim;
          const int kl = klen[j];
          if (m->dtype == MADE_BF16) {
            uint16_t* dst = (uint16_t*)host.data();
            for (int i = 0; i < kl; ++i) dst[frag_offset<bf16_t>(j, i, ly.k_chunks)] = host_f32_to_bf16(src[perm_prev[i]]);
          } else {
            float* dst = (float*)host.data();
            for (int i = 0; i < kl; ++i) dst[frag_offset<float>(j, i, ly.k_chunks)] = src[perm_prev[i]];
          }
        }
      };
      const int n_threads = n_w > ((size_t)1 << 24) ? 16 : 1;
      if (gather) {
        std::vector<std::thread> pool;
        const int per = (D + n_threads - 1) / n_threads;
        for (int i = 0; i < n_threads; ++i) {
          const int t0 = std::min(D, i * per), t1 = std::min(D, (i + 1) * per);
          if (t0 < t1) pool.emplace_back(fill_gather, t0, t1);
        }
        for (std::thread& th : pool) th.join();
      } else if (n_threads == 1) {
        fill_rows(0, ly.out_dim);
      } else {
        std::vector<std::thread> pool;
        const int per = (ly.out_dim + n_threads - 1) / n_threads;
        for (int i = 0; i < n_threads; ++i) {
          const int j0 = std::min(ly.out_dim, i * per), j1 = std::min(ly.out_dim, (i + 1) * per);
          if (j0 < j1) pool.emplace_back(fill_rows, j0, j1);
        }
        for (std::thread& th : pool) th.join();
      }
      std::vector<float> hb(ly.out_pad, 0.f);
      if (b && b[l])
        for (int j = 0; j < ly.out_dim; ++j) hb[j] = b[l][perm[j]];

      hipError_t he = hipMalloc(&ly.W, n_w * es);
      if (he == hipSuccess) he = hipMemcpy(ly.W, host.data(), n_w * es, hipMemcpyHostToDevice);
      if (he == hipSuccess) he = hipMalloc((void**)&ly.bias, ly.out_pad * sizeof(float));
      if (he == hipSuccess) he = hipMemcpy(ly.bias, hb.data(), ly.out_pad * sizeof(float), hipMemcpyHostToDevice);
      if (he == hipSuccess) he = hipMalloc((void**)&ly.tile_kend, ly.n_tiles * sizeof(int));
      if (he == hipSuccess)
        he = hipMemcpy(ly.tile_kend, ly.h_tile_kend.data(), ly.n_tiles * sizeof(int), hipMemcpyHostToDevice);
      if (he == hipSuccess && !is_out) {
        he = hipMalloc((void**)&ly.cnt_lt, m->cnt_lt[l].size() * sizeof(int));
        if (he == hipSuccess)
          he = hipMemcpy(ly.cnt_lt, m->cnt_lt[l].data(), m->cnt_lt[l].size() * sizeof(int), hipMemcpyHostToDevice);
        if (he == hipSuccess) he = hipMalloc((void**)&ly.slot_unit, perm.size() * sizeof(int));
        if (he == hipSuccess) he = hipMemcpy(ly.slot_unit, perm.data(), perm.size() * sizeof(int), hipMemcpyHostToDevice);
      }
      if (he != hipSuccess)
        rc = fail(he == hipErrorOutOfMemory ? MADE_ERR_NOMEM : MADE_ERR_HIP, "made_init: layer %d upload failed: %s", l,
                  hipGetErrorString(he));
      if (!is_out) {
        in_deg = out_deg;
        perm_prev = perm;
      }
    }
  } catch (const std::bad_alloc&) {
    rc = fail(MADE_ERR_NOMEM, "made_init: host allocation failed");
  }
  if (rc != MADE_OK) {
    made_free(m);
    return rc;
  }
  m->prof_ms.assign(L + 2, 0.0);
  m->prof_launches.assign(L + 2, 0);
  // The persistent kernel needs every workgroup resident at once: one per CU, if the device can do that.
  {
    int coop = 0, cus = 0, per_cu = 0;
    hipError_t pe = hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, m->device);
    if (pe == hipSuccess) pe = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, m->device);
    if (pe == hipSuccess)
      pe = m->dtype == MADE_BF16
               ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, persistent_sampler_kernel<bf16_t>, NW * 64, 0)
               : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, persistent_sampler_kernel<float>, NW * 64, 0);
    if (pe == hipSuccess && coop && per_cu >= 1 && C == 1 && L + 1 <= PERSIST_MAX_LAYERS) m->persist_grid = cus;
    // The XCD-local kernel wants two workgroups per compute unit resident at once on a chip of 8 XCDs.
    int per_cu_x = 0;
    if (pe == hipSuccess)
      pe = m->dtype == MADE_BF16
               ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_x, xcd_sampler_kernel<bf16_t>, NW * 64, 0)
               : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_x, xcd_sampler_kernel<float>, NW * 64, 0);
    if (pe == hipSuccess && per_cu_x >= 1 && cus >= XCDS && cus % XCDS == 0 && C == 1 && !m->real &&
        L + 1 <= PERSIST_MAX_LAYERS)
      m->xcd_grid = std::min(cus * std::min(per_cu_x, 2), XCDS * XCD_LINE);
    (void)hipGetLastError();
  }
  // The sample-resident kernel keeps one 32-sample row group of the input and of every hidden layer, the biases
  // and the mask tables in a workgroup's LDS, and the noise of up to RES_MAXT output tiles per wave in registers.
  bool res_fits = C == 1 && !m->real && L + 1 <= PERSIST_MAX_LAYERS && m->layers[L].n_tiles <= RES_MAXT * RES_W;
  for (int l = 0; l <= L; ++l) res_fits = res_fits && m->layers[l].n_tiles <= RES_TPW * RES_W;
  if (res_fits) {
    const int es = (int)elem_size(m);
    auto up16 = [](int v) { return (v + 15) & ~15; };
    int off = 0;
    m->res_lds_out.assign(L + 1, 0);
    m->res_lds_bias.assign(L + 1, 0);
    m->res_lds_kend.assign(L + 1, 0);
    m->res_lds_cnt.assign(L + 1, 0);
    m->res_lds_enc = off;
    off += m->layers[0].in_pad * RES_ROWS * es;
    for (int l = 0; l < L; ++l) {
      m->res_lds_out[l] = off;
      off += m->layers[l + 1].in_pad * RES_ROWS * es;
    }
    m->res_lds_clear = off;
    for (int l = 0; l <= L; ++l) {
      m->res_lds_bias[l] = off;
      off += m->layers[l].n_tiles * TILE * (int)sizeof(float);
      m->res_lds_kend[l] = off;
      off += up16(m->layers[l].n_tiles * (int)sizeof(int));
      if (l < L) {
        m->res_lds_cnt[l] = off;
        off += up16((D + 1) * (int)sizeof(int));
      }
    }
    const int statics = 2048;   // the kernel's own small LDS arrays
    if (off + statics <= 160 * 1024) {   // LDS of a gfx950 compute unit
      hipError_t le = m->dtype == MADE_BF16
               ? hipFuncSetAttribute((const void*)resident_sampler_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, off)
               : hipFuncSetAttribute((const void*)resident_sampler_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, off);
      if (le == hipSuccess) le = hipMalloc((void**)&m->res_ctr, 4 * sizeof(unsigned long long));
      if (le == hipSuccess) le = hipMemset(m->res_ctr, 0, 4 * sizeof(unsigned long long));
      if (le == hipSuccess) le = hipHostMalloc((void**)&m->res_host, 4 * sizeof(unsigned long long), hipHostMallocDefault);
      if (le == hipSuccess) m->res_lds_bytes = off;
    }
    (void)hipGetLastError();
  }
  *out = m;
  return MADE_OK;
}


// ------------------------------------------------------------------------------------------------
// masked convolutional model
// ------------------------------------------------------------------------------------------------
static void conv_group_of_feature(int F, std::vector<int>& grp) {
  const int s0 = (F + 2) / 3, s1 = (F - s0 + 1) / 2;
  grp.resize(F);
  for (int f = 0; f < F; ++f) grp[f] = f < s0 ? 0 : (f < s0 + s1 ? 1 : 2);
}

template <typename V>
static hipError_t upload(V** dev, const std::vector<V>& host) {
  hipError_t e = hipMalloc((void**)dev, std::max<size_t>(host.size(), 1) * sizeof(V));
  if (e == hipSuccess && !host.empty()) e = hipMemcpy(*dev, host.data(), host.size() * sizeof(V), hipMemcpyHostToDevice);
  return e;
}

extern "C" int made_conv_init(const made_conv_config* cfg, const float* const* W, const float* const* b,
                              made_model** out) {
  if (!out) return fail(MADE_ERR_ARG, "made_conv_init: out is NULL");
  *out = nullptr;
  if (!cfg || !W) return fail(MADE_ERR_ARG, "made_conv_init: NULL argument");
  if (cfg->W != 32) return fail(MADE_ERR_ARG, "made_conv_init: image width %d, only 32 is supported", cfg->W);
  if (cfg->H < 1 || cfg->H > 4096) return fail(MADE_ERR_ARG, "made_conv_init: H=%d out of range [1, 4096]", cfg->H);
  if (cfg->C != CAT_C) return fail(MADE_ERR_ARG, "made_conv_init: C=%d, only 256 classes are supported", cfg->C);
  if (cfg->dtype != MADE_F32 && cfg->dtype != MADE_BF16) return fail(MADE_ERR_ARG, "made_conv_init: unknown dtype %d", cfg->dtype);
  if (cfg->F != 64 && cfg->F != 128) return fail(MADE_ERR_ARG, "made_conv_init: F=%d, supported: 64, 128", cfg->F);
  if (cfg->k < 3 || cfg->k > CONV_MAX_K || cfg->k % 2 == 0)
    return fail(MADE_ERR_ARG, "made_conv_init: k=%d must be odd and <= %d", cfg->k, CONV_MAX_K);
  if (cfg->n_conv < 2 || cfg->n_conv > 62) return fail(MADE_ERR_ARG, "made_conv_init: n_conv=%d out of range [2, 62]", cfg->n_conv);
  for (int l = 0; l <= cfg->n_conv; ++l)
    if (!W[l]) return fail(MADE_ERR_ARG, "made_conv_init: W[%d] is NULL", l);

  made_model* m = new (std::nothrow) made_model();
  if (!m) return fail(MADE_ERR_NOMEM, "made_conv_init: host allocation failed");
  m->arch = 1;
  m->dtype = cfg->dtype;
  m->C = cfg->C;
  m->D = cfg->H * cfg->W * 3;
  m->L = cfg->n_conv;
  hipError_t e = hipGetDevice(&m->device);
  if (e != hipSuccess) {
    delete m;
    return fail(MADE_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  }
  ConvNet& cv = m->conv;
  cv.H = cfg->H;
  cv.F = cfg->F;
  cv.k = cfg->k;
  cv.n_conv = cfg->n_conv;
  const int F = cfg->F, k = cfg->k, mid = k / 2, kc = chunk_elems(m), kch = F / kc;
  std::vector<int> grp;
  conv_group_of_feature(F, grp);
  // visible taps: strictly above, or same row strictly left; the centre tap (partly visible) last
  std::vector<int> taps;
  std::vector<int> tap_kykx;
  for (int ky = 0; ky < k; ++ky)
    for (int kx = 0; kx < k; ++kx)
      if (ky < mid || (ky == mid && kx < mid)) {
        taps.push_back(ky - mid);
        taps.push_back(kx - mid);
        tap_kykx.push_back(ky * k + kx);
      }
  taps.push_back(0);
  taps.push_back(0);
  tap_kykx.push_back(mid * k + mid);
  cv.n_taps = (int)tap_kykx.size();
  const int64_t pixels = (int64_t)cfg->H * cfg->W;
  int rc = MADE_OK;
  try {
    e = upload(&cv.taps, taps);
    // first layer: [F x K0] with K index = tap * 3 + colour, fragment-major; centre tap: colour c visible iff
    // c < group(f)
    const int k0_chunks = (cv.n_taps * 3 + kc - 1) / kc;
    std::vector<uint8_t> w0((size_t)F * k0_chunks * kc * elem_size(m), 0);
    std::vector<float> b0(F, 0.f);
    int64_t nnz0 = 0;
    for (int f = 0; f < F; ++f)
      for (int t = 0; t < cv.n_taps; ++t)
        for (int c = 0; c < 3; ++c) {
          const bool centre = t == cv.n_taps - 1;
          if (centre && !(c < grp[f])) continue;
          const float v = W[0][((size_t)f * k * k + tap_kykx[t]) * 3 + c];
          const size_t off = m->dtype == MADE_BF16 ? frag_offset<bf16_t>(f, t * 3 + c, k0_chunks)
                                                   : frag_offset<float>(f, t * 3 + c, k0_chunks);
          if (m->dtype == MADE_BF16) ((uint16_t*)w0.data())[off] = host_f32_to_bf16(v);
          else ((float*)w0.data())[off] = v;
          nnz0++;
        }
    if (b && b[0]) b0.assign(b[0], b[0] + F);
    if (e == hipSuccess) e = hipMalloc(&cv.w0, w0.size());
    if (e == hipSuccess) e = hipMemcpy(cv.w0, w0.data(), w0.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = upload(&cv.b0, b0);
    m->nnz.push_back(nnz0 * pixels);
    // layers 1 .. n_conv-1: [F x n_taps*F] with K index = tap * F + input channel; centre tap: in group <= out group
    const int k_chunks = cv.n_taps * kch;
    for (int l = 1; l < cfg->n_conv && e == hipSuccess; ++l) {
      const size_t n_w = (size_t)F * cv.n_taps * F;
      std::vector<uint8_t> host(n_w * elem_size(m), 0);
      int64_t nnz = 0;
      for (int f = 0; f < F; ++f)
        for (int t = 0; t < cv.n_taps; ++t)
          for (int ci = 0; ci < F; ++ci) {
            const bool centre = t == cv.n_taps - 1;
            if (centre && !(grp[ci] <= grp[f])) continue;
            const float v = W[l][((size_t)f * k * k + tap_kykx[t]) * F + ci];
            const size_t off = m->dtype == MADE_BF16 ? frag_offset<bf16_t>(f, t * F + ci, k_chunks)
                                                     : frag_offset<float>(f, t * F + ci, k_chunks);
            if (m->dtype == MADE_BF16) ((uint16_t*)host.data())[off] = host_f32_to_bf16(v);
            else ((float*)host.data())[off] = v;
            nnz++;
          }
      void* dw = nullptr;
      e = hipMalloc(&dw, host.size());
      if (e == hipSuccess) e = hipMemcpy(dw, host.data(), host.size(), hipMemcpyHostToDevice);
      cv.w.push_back(dw);
      std::vector<float> hb(F, 0.f);
      if (b && b[l]) hb.assign(b[l], b[l] + F);
      float* db = nullptr;
      if (e == hipSuccess) e = upload(&db, hb);
      cv.bias.push_back(db);
      m->nnz.push_back(nnz * pixels);
    }
    // head: rows c*256 + class read features of group <= c (a prefix, features are ordered by group)
    if (e == hipSuccess) {
      const int rows = 3 * CAT_C;
      std::vector<uint8_t> host((size_t)rows * F * elem_size(m), 0);
      std::vector<int> kend(rows / TILE, 0);
      int64_t nnz = 0;
      for (int r = 0; r < rows; ++r)
        for (int f = 0; f < F; ++f) {
          if (!(grp[f] <= r / CAT_C)) continue;
          const float v = W[cfg->n_conv][(size_t)r * F + f];
          const size_t off = m->dtype == MADE_BF16 ? frag_offset<bf16_t>(r, f, kch) : frag_offset<float>(r, f, kch);
          if (m->dtype == MADE_BF16) ((uint16_t*)host.data())[off] = host_f32_to_bf16(v);
          else ((float*)host.data())[off] = v;
          kend[r / TILE] = std::max(kend[r / TILE], round_up(f + 1, kc));
          nnz++;
        }
      e = hipMalloc(&cv.w_head, host.size());
      if (e == hipSuccess) e = hipMemcpy(cv.w_head, host.data(), host.size(), hipMemcpyHostToDevice);
      std::vector<float> hb(rows, 0.f);
      if (b && b[cfg->n_conv]) hb.assign(b[cfg->n_conv], b[cfg->n_conv] + rows);
      if (e == hipSuccess) e = upload(&cv.b_head, hb);
      if (e == hipSuccess) e = upload(&cv.head_tile_kend, kend);
      m->nnz.push_back(nnz * pixels);
    }
    if (e != hipSuccess)
      rc = fail(e == hipErrorOutOfMemory ? MADE_ERR_NOMEM : MADE_ERR_HIP, "made_conv_init: upload failed: %s",
                hipGetErrorString(e));
  } catch (const std::bad_alloc&) {
    rc = fail(MADE_ERR_NOMEM, "made_conv_init: host allocation failed");
  }
  if (rc != MADE_OK) {
    made_free(m);
    return rc;
  }
  m->prof_ms.assign(m->L + 2, 0.0);
  m->prof_launches.assign(m->L + 2, 0);
  *out = m;
  return MADE_OK;
}

// ------------------------------------------------------------------------------------------------
// launches
// ------------------------------------------------------------------------------------------------
struct RowSet {            // which samples a pass covers
  const int* rows;         // device list or NULL (identity)
  const int* n_rows_ptr;   // device count or NULL
  int n_rows;              // host-side upper bound (grid size) and value when n_rows_ptr is NULL
  const uint8_t* x = nullptr;   // current symbols [N, D]: what a one-hot first layer reads instead of the scalar encoding
  int pos_base = 0;             // first sample of the chain the list belongs to (see LayerArgs::pos_base)
};

struct SampleIO {          // what the sampling epilogue reads and writes
  const float* noise;
  uint8_t* x;              // symbols; for a model with real states this is a float [N, D] buffer
  int t_lo, t_hi;
  RetireArgs retire;       // retire.enabled = 0: no stop test after this pass (sequential sampling)
  const int* t_first_ptr = nullptr;   // 256-class output kernel: first position to evaluate / where the lowest changed
  int* first_changed = nullptr;       // position is recorded (see CatArgs)
  unsigned* lazy_mask = nullptr;   // Bernoulli MLP: changed rows go here as bits and the next pass derives its list from
                                   // them (see DeriveArgs); retire.enabled is 0 then
};

template <typename T, int EPI>
static void launch_layer_t(LayerArgs a, int n_tiles, int row_tiles, hipStream_t s) {
  a.n_launch_tiles = n_tiles;
  a.row_tiles = row_tiles;
  const int groups = (n_tiles + XCDS - 1) / XCDS;     // tile groups of 8, one tile per XCD
  hipLaunchKernelGGL((masked_layer_kernel<T, EPI>), dim3(groups * XCDS * row_tiles), dim3(NW * 64), 0, s, a);
}

static void prof_mark(made_model* m, int layer, bool after, hipStream_t s) {
  if (!m->profiling) return;
  const size_t pair = after ? m->ev_layer.size() - 1 : m->ev_layer.size();
  if (!after) {
    while (m->ev_pool.size() < 2 * (pair + 1)) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) { m->profiling = false; return; }
      m->ev_pool.push_back(e);
    }
    m->ev_layer.push_back(layer);
  }
  (void)hipEventRecord(m->ev_pool[2 * pair + (after ? 1 : 0)], s);
}

// after the stream has been synchronised: fold the event pairs of this call into per-layer sums
static void prof_collect(made_model* m) {
  std::fill(m->prof_ms.begin(), m->prof_ms.end(), 0.0);
  std::fill(m->prof_launches.begin(), m->prof_launches.end(), 0);
  for (size_t i = 0; i < m->ev_layer.size(); ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, m->ev_pool[2 * i], m->ev_pool[2 * i + 1]) == hipSuccess) {
      m->prof_ms[m->ev_layer[i]] += ms;
      m->prof_launches[m->ev_layer[i]]++;
    }
  }
  m->ev_layer.clear();
}

template <typename T, int EPI, int W>
static void launch_big_t(LayerArgs a, int n_tiles, int n_rows_max, hipStream_t s) {
  constexpr int BIG_T = 2 * W, BIG_ROWS = BIG_T * TILE;   // tiles / samples per workgroup and dimension
  a.n_launch_tiles = n_tiles;
  a.row_tiles = (n_rows_max + BIG_ROWS - 1) / BIG_ROWS;
  const int big_cols = (n_tiles + BIG_T - 1) / BIG_T;
  const int pair_cols = (big_cols + 1) / 2;                // a workgroup takes a long and a short column of unit tiles
  a.big_by_rows = a.row_tiles >= pair_cols;
  const int groups = ((a.big_by_rows ? a.row_tiles : pair_cols) + XCDS - 1) / XCDS;
  const int other = a.big_by_rows ? pair_cols : a.row_tiles;
  hipLaunchKernelGGL((masked_layer_big_kernel<T, EPI, W>), dim3(groups * XCDS * other), dim3(256), 0, s, a);   // (static LDS: 128 / 64 KB)
}

template <int EPI>
static void launch_layer(made_model* m, int layer, const LayerArgs& a, int n_tiles, int row_tiles, hipStream_t s) {
  prof_mark(m, layer, false, s);
  // (launches that start behind cached partial sums cover few units: they stay on the 32 x 32 tiles, whose grids are
  // the larger ones there, and only that kernel takes k_begin / partial)
  const bool small_only = a.partial != nullptr || a.k_begin > 0;
  const bool big = !small_only && a.n_rows >= m->big_batch && (EPI == EPI_RELU || m->big_output);
  const bool mid = !small_only && !big && a.n_rows >= m->mid_batch;
  if (m->dtype == MADE_BF16) {
    if (big) launch_big_t<bf16_t, EPI, 4>(a, n_tiles, a.n_rows, s);
    else if (mid) launch_big_t<bf16_t, EPI, 2>(a, n_tiles, a.n_rows, s);
    else launch_layer_t<bf16_t, EPI>(a, n_tiles, row_tiles, s);
  } else {
    if (big) launch_big_t<float, EPI, 4>(a, n_tiles, a.n_rows, s);
    else if (mid) launch_big_t<float, EPI, 2>(a, n_tiles, a.n_rows, s);
    else launch_layer_t<float, EPI>(a, n_tiles, row_tiles, s);
  }
  prof_mark(m, layer, true, s);
}

static LayerArgs base_args(const made_model* m, int l, const void* A, const RowSet& rs) {
  const Layer& ly = m->layers[l];
  LayerArgs a;
  memset(&a, 0, sizeof a);
  a.A = A;
  a.W = ly.W;
  a.k_chunks = ly.k_chunks;
  a.bias = ly.bias;
  a.tile_kend = ly.tile_kend;
  a.k_cap = ly.in_pad;
  a.tile_begin = 0;
  a.rows = rs.rows;
  a.n_rows_ptr = rs.n_rows_ptr;
  a.n_rows = rs.n_rows;
  a.n_rows_pad = round_up(std::max(rs.n_rows, 1), 2 * TILE);
  a.n_cols = ly.out_dim;
  a.pos_base = rs.pos_base;
  return a;
}

// Hidden layers for the samples of `rs`.  unit_limit[l] < 0 means the whole layer; otherwise only the
// first unit_limit[l] (degree-sorted) units are evaluated, reading only the first in_limit inputs.
// unit_first (optional): units below unit_first[l] are frozen -- their inputs are final and their activations
// are already in the layer's buffer from an earlier pass -- so only the tiles from there on are evaluated.
// by_pos: hidden activations are stored by position in the active list (see LayerArgs::a_by_pos); the caller
// then runs the output layer the same way.  Only for whole-layer passes on the 32 x 32 tile kernels.
static bool hidden_by_position(const made_model* m, const RowSet& rs, bool limited) {
  return m->arch == 0 && !limited && !m->onehot && (m->C == 1 || m->real) && rs.rows != nullptr &&
         rs.n_rows < std::min(m->big_batch, m->mid_batch);
}

// Where a forward pass keeps the network input and the hidden activations: the model's workspace (NULL), or
// buffers of the caller's choosing (the entry point that must not allocate passes pieces of a static array).
struct ActBuffers {
  void* enc;
  void* act[64];         // (made_init admits at most 64 hidden layers)
};

// Cached partial sums of a GS-Jacobi block (see enqueue_pass): layer l multiplies only the inputs from k_first[l] on
// and adds sums[l] (fp32 [sample, out_pad]) for the inputs before them.  Index L is the output layer.
struct PartialSums {
  const int* k_first;
  float* const* sums;
};

static int run_hidden(made_model* m, const RowSet& rs, const int* unit_limit, int in_limit0, hipStream_t s,
                      const int* unit_first = nullptr, bool by_pos = false, const ActBuffers* buf = nullptr,
                      const PartialSums* ps = nullptr, const DeriveArgs* derive = nullptr, int first_layer = 0) {
  const int row_tiles = (rs.n_rows + TILE - 1) / TILE;
  const int kc = chunk_elems(m);
  int in_limit = in_limit0;
  for (int l = first_layer; l < m->L; ++l) {   // (first_layer = 1: the call's set-up kernel has written layer 0's activations)
    const Layer& ly = m->layers[l];
    LayerArgs a = base_args(m, l, l == 0 ? (buf ? buf->enc : m->ws.enc) : (buf ? buf->act[l - 1] : m->ws.act[l - 1]), rs);
    a.out = buf ? buf->act[l] : m->ws.act[l];
    a.out_chunks = m->layers[l + 1].k_chunks;
    int tiles = ly.n_tiles;
    if (unit_limit && unit_limit[l] >= 0) tiles = std::min(tiles, (unit_limit[l] + TILE - 1) / TILE);
    if (in_limit >= 0) a.k_cap = std::min(ly.in_pad, round_up(in_limit, kc));
    if (unit_first) a.tile_begin = std::min(tiles, unit_first[l] / TILE);
    if (ps && ps->k_first[l] > 0) {
      a.k_begin = ps->k_first[l];
      a.partial = ps->sums[l];
      a.ld_partial = ly.out_pad;
    }
    a.a_by_pos = by_pos && l > 0;
    a.out_by_pos = by_pos;
    if (l == 0 && derive) a.derive = *derive;
    if (l == 0 && m->onehot) {
      if (!rs.x) return fail(MADE_ERR_ARG, "internal: a one-hot first layer needs the symbols");
      if (rs.n_rows > 65535) return fail(MADE_ERR_ARG, "one-hot input: at most 65535 samples per call");
      if (tiles - a.tile_begin > 0) {
        OnehotArgs g;
        g.Wg = ly.W;
        g.bias = ly.bias;
        g.x = rs.x;
        g.rows = rs.rows;
        g.n_rows_ptr = rs.n_rows_ptr;
        g.n_rows = rs.n_rows;
        g.cnt_lt = ly.cnt_lt;
        g.D = m->D;
        g.C = m->C;
        g.pitch = ly.out_pad;
        g.t_end = in_limit >= 0 ? std::min(in_limit, m->D) : m->D;
        g.unit_begin = a.tile_begin * TILE;
        g.unit_end = tiles * TILE;
        g.out = a.out;
        g.out_chunks = a.out_chunks;
        const int chunks = (g.unit_end - g.unit_begin + ONEHOT_UNITS - 1) / ONEHOT_UNITS;
        prof_mark(m, 0, false, s);
        if (m->dtype == MADE_BF16)
          hipLaunchKernelGGL(onehot_first_layer_kernel<bf16_t>, dim3((chunks + 1) / 2, std::max(rs.n_rows, 1)), dim3(ONEHOT_THREADS), 0, s, g);
        else
          hipLaunchKernelGGL(onehot_first_layer_kernel<float>, dim3((chunks + 1) / 2, std::max(rs.n_rows, 1)), dim3(ONEHOT_THREADS), 0, s, g);
        prof_mark(m, 0, true, s);
        m->stats[2]++;
      }
    } else if (tiles - a.tile_begin > 0) {
      launch_layer<EPI_RELU>(m, l, a, tiles - a.tile_begin, row_tiles, s);
      m->stats[2]++;
    }
    in_limit = (unit_limit && unit_limit[l] >= 0) ? unit_limit[l] : -1;
  }
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

// Output layer + draw for positions [t_lo, t_hi).  whole = evaluate every output tile regardless.
static int run_output_sample(made_model* m, const RowSet& rs, const SampleIO& io, bool whole, int k_limit,
                             hipStream_t s, bool by_pos = false, const PartialSums* ps = nullptr) {
  const Layer& ly = m->layers[m->L];
  const int row_tiles = (rs.n_rows + TILE - 1) / TILE;
  const int kc = chunk_elems(m);
  LayerArgs a = base_args(m, m->L, m->ws.act[m->L - 1], rs);
  a.a_by_pos = by_pos;
  if (k_limit >= 0) a.k_cap = std::min(ly.in_pad, round_up(k_limit, kc));
  const int C = m->C;
  int tile_lo = 0, tile_hi = ly.n_tiles;
  if (!whole) {
    tile_lo = (io.t_lo * C) / TILE;
    tile_hi = (io.t_hi * C + TILE - 1) / TILE;
  }
  a.tile_begin = tile_lo;
  if (m->real) {
    a.noise = io.noise;
    a.xr = (float*)io.x;
    a.eps = m->call_eps;
    a.enc = m->ws.enc;
    a.enc_chunks = m->layers[0].k_chunks;
    a.changed = m->ws.changed;
    a.D = m->D;
    a.t_lo = io.t_lo;
    a.t_hi = io.t_hi;
    a.retire = io.retire;
    prof_mark(m, m->L, false, s);
    if (m->dtype == MADE_BF16) launch_layer_t<bf16_t, EPI_LOGISTIC>(a, tile_hi - tile_lo, row_tiles, s);
    else launch_layer_t<float, EPI_LOGISTIC>(a, tile_hi - tile_lo, row_tiles, s);
    prof_mark(m, m->L, true, s);
    m->stats[2]++;
  } else if (C == 1) {
    a.noise = io.noise;
    a.x = io.x;
    a.enc = m->ws.enc;
    a.enc_chunks = m->layers[0].k_chunks;
    a.changed = m->ws.changed;
    a.D = m->D;
    a.t_lo = io.t_lo;
    a.t_hi = io.t_hi;
    a.retire = io.retire;
    a.lazy_mask = io.lazy_mask;
    a.io_aligned = (m->D % 16 == 0) && ((uintptr_t)io.noise % 16 == 0) && ((uintptr_t)io.x % 16 == 0);
    if (ps && ps->k_first[m->L] > 0) {
      a.k_begin = ps->k_first[m->L];
      a.partial = ps->sums[m->L];
      a.ld_partial = ly.out_pad;
    }
    launch_layer<EPI_BERNOULLI>(m, m->L, a, tile_hi - tile_lo, row_tiles, s);
    m->stats[2]++;
  } else if (C == CAT_C && m->fused_categorical) {
    CatArgs c;
    memset(&c, 0, sizeof c);
    c.A = a.A;
    c.W = a.W;
    c.k_chunks = a.k_chunks;
    c.bias = a.bias;
    c.tile_kend = a.tile_kend;
    c.k_cap = a.k_cap;
    c.rows = rs.rows;
    c.n_rows_ptr = rs.n_rows_ptr;
    c.n_rows = rs.n_rows;
    c.noise = io.noise;
    c.x = io.x;
    c.enc = m->ws.enc;
    c.enc_chunks = m->layers[0].k_chunks;
    c.changed = m->ws.changed;
    c.D = m->D;
    c.t_lo = io.t_lo;
    c.t_hi = io.t_hi;
    c.t_begin = whole ? 0 : io.t_lo;
    c.n_pos = whole ? m->D : io.t_hi - io.t_lo;
    c.pair_tiles = (rs.n_rows + 2 * TILE - 1) / (2 * TILE);
    c.t_first_ptr = io.t_first_ptr;
    c.first_changed = io.first_changed;
    c.retire = io.retire;
    prof_mark(m, m->L, false, s);
    if (m->dtype == MADE_BF16)
      hipLaunchKernelGGL((categorical_output_kernel<bf16_t>), dim3(c.n_pos * c.pair_tiles), dim3(CAT_WAVES * 64), 0, s, c);
    else
      hipLaunchKernelGGL((categorical_output_kernel<float>), dim3(c.n_pos * c.pair_tiles), dim3(CAT_WAVES * 64), 0, s, c);
    prof_mark(m, m->L, true, s);
    m->stats[2]++;
  } else {
    a.out = m->ws.zbuf;
    a.ldo = m->D * C;
    launch_layer<EPI_LOGITS>(m, m->L, a, tile_hi - tile_lo, row_tiles, s);
    const int span = io.t_hi - io.t_lo;
    const long long waves = (long long)rs.n_rows * span;
    const int blocks = (int)((waves + 3) / 4);
    if (m->dtype == MADE_BF16)
      hipLaunchKernelGGL((gumbel_argmax_kernel<bf16_t>), dim3(blocks), dim3(256), 0, s, m->ws.zbuf, m->D * C, io.noise,
                         io.x, (bf16_t*)m->ws.enc, m->layers[0].k_chunks, m->ws.changed, rs.rows, rs.n_rows_ptr,
                         rs.n_rows, m->D, C, io.t_lo, io.t_hi, io.retire);
    else
      hipLaunchKernelGGL((gumbel_argmax_kernel<float>), dim3(blocks), dim3(256), 0, s, m->ws.zbuf, m->D * C, io.noise,
                         io.x, (float*)m->ws.enc, m->layers[0].k_chunks, m->ws.changed, rs.rows, rs.n_rows_ptr,
                         rs.n_rows, m->D, C, io.t_lo, io.t_hi, io.retire);
    m->stats[2] += 2;
  }
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

// One pass of the convolutional network over ALL images of the batch (converged images are recomputed; their
// symbols cannot change), then the fused head: Gumbel-max draw of the states in [state_lo, state_hi).
static void launch_conv_trunk(made_model* m, const uint8_t* x, int N, const int* dirty_lo, int row_hi, hipStream_t s,
                              const void** last_act, const int* row_hi_of = nullptr) {
  ConvNet& cv = m->conv;
  const int kch = cv.F / chunk_elems(m);
  const int ft = cv.F / 32;
  ConvFirstArgs fa;
  memset(&fa, 0, sizeof fa);
  fa.win = ConvWindow{dirty_lo, row_hi, row_hi_of};
  fa.x = x;
  fa.w = cv.w0;
  fa.bias = cv.b0;
  fa.out = cv.act[0];
  fa.out_chunks = kch;
  fa.N = N;
  fa.H = cv.H;
  prof_mark(m, 0, false, s);
  {
    const dim3 grid(N * cv.H), block(ft * 64);
#define JM_FIRST_K(T, FT)                                                                                 \
  do {                                                                                                   \
    if (cv.k == 3) hipLaunchKernelGGL((conv_first_kernel<T, FT, 3>), grid, block, 0, s, fa);             \
    else if (cv.k == 5) hipLaunchKernelGGL((conv_first_kernel<T, FT, 5>), grid, block, 0, s, fa);        \
    else hipLaunchKernelGGL((conv_first_kernel<T, FT, 7>), grid, block, 0, s, fa);                       \
  } while (0)
    if (m->dtype == MADE_BF16) {
      if (ft == 4) JM_FIRST_K(bf16_t, 4); else JM_FIRST_K(bf16_t, 2);
    } else {
      if (ft == 4) JM_FIRST_K(float, 4); else JM_FIRST_K(float, 2);
    }
#undef JM_FIRST_K
  }
  prof_mark(m, 0, true, s);
  m->stats[2]++;
  const int mid = cv.k / 2;
  const int wg_rows = cv.wg_rows;
  // padded input rows in fragment order; the epilogue re-uses the space for four 32 x 33 float patches
  const size_t lds = std::max<size_t>((size_t)(wg_rows + mid) * kch * 8 * (32 + 2 * mid) * 16, (size_t)4 * TILE * (TILE + 1) * 4);
  const int grid = N * ((cv.H + wg_rows - 1) / wg_rows);
  for (int l = 1; l < cv.n_conv; ++l) {
    ConvLayerArgs a;
    memset(&a, 0, sizeof a);
    a.win = ConvWindow{dirty_lo, row_hi, row_hi_of};
    a.in = cv.act[l - 1];
    a.w = cv.w[l - 1];
    a.bias = cv.bias[l - 1];
    a.out = cv.act[l];
    a.N = N;
    a.H = cv.H;
    prof_mark(m, l, false, s);
#define JM_LAUNCH_CONV(T, FT, KS, WR)                                                                              \
  do {                                                                                                            \
    static size_t configured = 0;                                                                                 \
    if (lds > configured) {                                                                                       \
      (void)hipFuncSetAttribute((const void*)conv_layer_kernel<T, FT, KS, WR>,                                    \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                            \
      configured = lds;                                                                                           \
    }                                                                                                             \
    hipLaunchKernelGGL((conv_layer_kernel<T, FT, KS, WR>), dim3(grid), dim3(256), lds, s, a);                     \
  } while (0)
#define JM_CONV_ROWS(T, FT, KS) do { if (wg_rows == 4) JM_LAUNCH_CONV(T, FT, KS, 4); else JM_LAUNCH_CONV(T, FT, KS, 2); } while (0)
#define JM_CONV_K(T, FT)                                                                                           \
  do {                                                                                                            \
    if (cv.k == 3) JM_CONV_ROWS(T, FT, 3); else if (cv.k == 5) JM_CONV_ROWS(T, FT, 5); else JM_CONV_ROWS(T, FT, 7); \
  } while (0)
    if (m->dtype == MADE_BF16) {
      if (ft == 4) JM_CONV_K(bf16_t, 4); else JM_CONV_K(bf16_t, 2);
    } else {
      if (ft == 4) JM_CONV_K(float, 4); else JM_CONV_K(float, 2);
    }
#undef JM_CONV_K
#undef JM_CONV_ROWS
#undef JM_LAUNCH_CONV
    prof_mark(m, l, true, s);
    m->stats[2]++;
  }
  *last_act = cv.act[cv.n_conv - 1];
}

static void launch_conv_head(made_model* m, const ConvHeadArgs& c, hipStream_t s);

static int run_conv_pass(made_model* m, int N, const SampleIO& io, bool first_pass, bool whole_network,
                         hipStream_t s) {
  ConvNet& cv = m->conv;
  const void* last = nullptr;
  const int row_lo = io.t_lo / (32 * 3), row_hi = (io.t_hi - 1) / (32 * 3);   // rows holding the states drawn
  int* dirty_lo = whole_network ? nullptr : cv.win;
  launch_conv_trunk(m, io.x, N, dirty_lo, whole_network ? cv.H - 1 : row_hi, s, &last);
  ConvHeadArgs c;
  memset(&c, 0, sizeof c);
  c.A = last;
  c.W = cv.w_head;
  c.bias = cv.b_head;
  c.tile_kend = cv.head_tile_kend;
  c.noise = io.noise;
  c.x = io.x;
  c.changed = m->ws.changed;
  c.N = N;
  c.H = cv.H;
  c.state_lo = io.t_lo;
  c.state_hi = io.t_hi;
  // one workgroup per CU in all (3 colours x 85; the kernel runs one wave per SIMD); workgroup (colour, group)
  // walks over the pixel rows group, group + groups, ..., its 4 waves splitting the classes of each row
  c.groups = std::max(1, std::min(N * cv.H, 85));
  if (!whole_network) {
    c.dirty_lo = cv.win;
    c.first_changed = cv.win + cv.win_pad;
    c.win_done = cv.win + (size_t)cv.win_pad * (1 + CHG);
    c.rows_stat = cv.rows_stat;
    c.row_lo = row_lo;
    c.row_hi = row_hi;
    c.first_pass = first_pass ? 1 : 0;
  }
  c.retire = io.retire;
  launch_conv_head(m, c, s);
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

static void launch_conv_head(made_model* m, const ConvHeadArgs& c, hipStream_t s) {
  ConvNet& cv = m->conv;
  prof_mark(m, m->L, false, s);
#define JM_LAUNCH_HEAD(T, FT) hipLaunchKernelGGL((conv_head_kernel<T, FT>), dim3(3 * c.groups), dim3(256), 0, s, c)
  if (m->dtype == MADE_BF16) {
    if (cv.F == 128) JM_LAUNCH_HEAD(bf16_t, 4); else JM_LAUNCH_HEAD(bf16_t, 2);
  } else {
    if (cv.F == 128) JM_LAUNCH_HEAD(float, 4); else JM_LAUNCH_HEAD(float, 2);
  }
#undef JM_LAUNCH_HEAD
  prof_mark(m, m->L, true, s);
  m->stats[2]++;
}

static int launch_init_state(made_model* m, const uint8_t* x_init, uint8_t* x, int N, hipStream_t s,
                             const CallReset* reset_in = nullptr, void* enc_buf = nullptr) {
  void* const enc = enc_buf ? enc_buf : m->ws.enc;
  CallReset reset;
  memset(&reset, 0, sizeof reset);
  if (reset_in) reset = *reset_in;
  const size_t total = (size_t)N * m->D;
  const int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
  if (m->arch == 1) {   // the first convolution reads the symbols themselves
    if (x) {
      ConvNet& cv = m->conv;
      hipLaunchKernelGGL(copy_symbols_kernel, dim3(blocks), dim3(256), 0, s, x_init, x, total);
      hipLaunchKernelGGL(conv_reset_window_kernel, dim3((N + 255) / 256), dim3(256), 0, s, cv.win,
                         cv.win + cv.win_pad, N, cv.win + (size_t)cv.win_pad * (1 + CHG), cv.rows_stat);
      m->stats[2]++;
    }
    m->stats[2]++;
    HIP_TRY(hipGetLastError());
    return MADE_OK;
  }
  if (m->real) {
    if (m->dtype == MADE_BF16)
      hipLaunchKernelGGL((init_state_real_kernel<bf16_t>), dim3(blocks), dim3(256), 0, s, (const float*)x_init, (float*)x,
                         (bf16_t*)enc, m->layers[0].k_chunks, N, m->D, reset);
    else
      hipLaunchKernelGGL((init_state_real_kernel<float>), dim3(blocks), dim3(256), 0, s, (const float*)x_init, (float*)x,
                         (float*)enc, m->layers[0].k_chunks, N, m->D, reset);
    m->stats[2]++;
    HIP_TRY(hipGetLastError());
    return MADE_OK;
  }
  if (m->dtype == MADE_BF16)
    hipLaunchKernelGGL((init_state_kernel<bf16_t>), dim3(blocks), dim3(256), 0, s, x_init, x, (bf16_t*)enc,
                       m->layers[0].k_chunks, N, m->D, m->C, reset);
  else
    hipLaunchKernelGGL((init_state_kernel<float>), dim3(blocks), dim3(256), 0, s, x_init, x, (float*)enc,
                       m->layers[0].k_chunks, N, m->D, m->C, reset);
  m->stats[2]++;
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

static int check_call(made_model* m, const void* noise, int32_t N, const void* x_out, const char* who,
                      bool real_entry = false) {
  if (!m) return fail(MADE_ERR_ARG, "%s: model is NULL", who);
  if (m->real != real_entry)
    return fail(MADE_ERR_ARG, m->real ? "%s: the model has real states, use the *_real entry points"
                                      : "%s: the model has discrete states", who);
  if (N < 0) return fail(MADE_ERR_ARG, "%s: N=%d is negative", who, N);
  if (N > (1 << 22)) return fail(MADE_ERR_ARG, "%s: N=%d exceeds 2^22", who, N);
  if (N > 0 && (!noise || !x_out)) return fail(MADE_ERR_ARG, "%s: NULL noise or output pointer", who);
  if (m->poisoned)
    return fail(MADE_ERR_HIP, "%s: an earlier call on this model timed out waiting for the device; synchronise the "
                              "device, release the model with made_free and build a new one", who);
  HIP_TRY(hipSetDevice(m->device));
  return MADE_OK;
}

// ------------------------------------------------------------------------------------------------
// entry points
// ------------------------------------------------------------------------------------------------
extern "C" int made_forward_logits(made_model* m, const uint8_t* x, int32_t N, float* logits, void* stream) {
  TRY(check_call(m, x, N, logits, "made_forward_logits"));
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  const bool was_profiling = m->profiling;
  m->profiling = false;  // this call does not wait for the stream, so it cannot read event times
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, false));
  if (m->arch == 1) {
    const void* last = nullptr;
    launch_conv_trunk(m, x, N, nullptr, m->conv.H - 1, s, &last);
    // the 1 x 1 head is a plain layer over pixels: logits[pixel][colour * 256 + class]
    ConvNet& cv = m->conv;
    LayerArgs a;
    memset(&a, 0, sizeof a);
    a.A = last;
    a.W = cv.w_head;
    a.k_chunks = cv.F / chunk_elems(m);
    a.bias = cv.b_head;
    a.tile_kend = cv.head_tile_kend;
    a.k_cap = cv.F;
    a.n_rows = N * cv.H * 32;
    a.n_rows_pad = round_up(a.n_rows, 2 * TILE);
    a.n_cols = 3 * CAT_C;
    a.out = logits;
    a.ldo = 3 * CAT_C;
    const int big_saved = m->big_batch, mid_saved = m->mid_batch;
    m->big_batch = m->mid_batch = 1 << 30;    // (the head has only 768 outputs: always the 32 x 32 tiles)
    launch_layer<EPI_LOGITS>(m, m->L, a, 3 * CAT_C / TILE, (a.n_rows + TILE - 1) / TILE, s);
    m->big_batch = big_saved;
    m->mid_batch = mid_saved;
    m->profiling = was_profiling;
    HIP_TRY(hipGetLastError());
    return MADE_OK;
  }
  TRY(launch_init_state(m, x, nullptr, N, s));
  RowSet rs{nullptr, nullptr, N, x};
  TRY(run_hidden(m, rs, nullptr, -1, s));
  LayerArgs a = base_args(m, m->L, m->ws.act[m->L - 1], rs);
  a.out = logits;
  a.ldo = m->D * m->C;
  launch_layer<EPI_LOGITS>(m, m->L, a, m->layers[m->L].n_tiles, (N + TILE - 1) / TILE, s);
  m->profiling = was_profiling;
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

// One pass over the whole network like made_forward_logits, for callers that cannot allocate: network input and
// hidden activations live in this device's copy of the static `scratch` array instead of the model's workspace,
// and nothing here calls hipMalloc / hipFree or waits for the device.  The used part of the array is cleared
// first (by a kernel, so that the call may be captured into a graph): the masked weights are zero in the K
// padding of a layer, but what an earlier call of another model left there could be Inf or NaN.
extern "C" int made_forward_logits_noalloc(made_model* m, const uint8_t* x, int32_t N, float* logits, void* stream) {
  if (!m) return fail(MADE_ERR_ARG, "made_forward_logits_noalloc: model is NULL");
  if (m->arch != 0 || m->real)
    return fail(MADE_ERR_ARG, "made_forward_logits_noalloc: only masked MLPs with discrete states are supported");
  if (N < 0) return fail(MADE_ERR_ARG, "made_forward_logits_noalloc: N=%d is negative", N);
  if (N > 0 && (!x || !logits)) return fail(MADE_ERR_ARG, "made_forward_logits_noalloc: NULL symbols or logits pointer");
  if (m->poisoned) return fail(MADE_ERR_HIP, "made_forward_logits_noalloc: an earlier call on this model timed out");
  if (N == 0) return MADE_OK;
  // layout: [enc | act 0 | ... | act L-1], each n_pad rows of the layer's padded input width, 256-byte aligned
  const size_t es = elem_size(m);
  const size_t n_pad = (size_t)round_up(N, 2 * TILE);
  size_t per_row = 0;
  for (int l = 0; l <= m->L; ++l) per_row += (size_t)m->layers[l].in_pad * es;
  const size_t need = n_pad * per_row;                     // (every piece is a multiple of 64 rows x 128 bytes)
  if (need > NOALLOC_SCRATCH_BYTES)
    return fail(MADE_ERR_ARG, "made_forward_logits_noalloc: N=%d needs %zu bytes of scratch memory, the static array "
                              "holds %zu (at most %zu samples of this model per call)", N, need, NOALLOC_SCRATCH_BYTES,
                (NOALLOC_SCRATCH_BYTES / per_row) / (2 * TILE) * (2 * TILE));
  HIP_TRY(hipSetDevice(m->device));
  void* base = nullptr;
  {
    const hipError_t e = scratch_address(m->device, &base);   // (looked up in made_init; a table read here)
    if (e != hipSuccess) return fail(MADE_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
  }
  hipStream_t s = (hipStream_t)stream;
  ActBuffers buf;
  memset(&buf, 0, sizeof buf);
  size_t off = 0;
  buf.enc = (unsigned char*)base + off;
  off += n_pad * m->layers[0].in_pad * es;
  for (int l = 0; l < m->L; ++l) {
    buf.act[l] = (unsigned char*)base + off;
    off += n_pad * m->layers[l + 1].in_pad * es;
  }
  const bool was_profiling = m->profiling;
  m->profiling = false;
  {
    const size_t n16 = need / 16;
    const int blocks = (int)std::min<size_t>((n16 + 255) / 256, 2048);
    hipLaunchKernelGGL(zero_fill_kernel, dim3(blocks), dim3(256), 0, s, (uint4*)base, n16);
  }
  int rc = launch_init_state(m, x, nullptr, N, s, nullptr, buf.enc);
  RowSet rs{nullptr, nullptr, N, x};
  if (rc == MADE_OK) rc = run_hidden(m, rs, nullptr, -1, s, nullptr, false, &buf);
  if (rc == MADE_OK) {
    LayerArgs a = base_args(m, m->L, buf.act[m->L - 1], rs);
    a.out = logits;
    a.ldo = m->D * m->C;
    launch_layer<EPI_LOGITS>(m, m->L, a, m->layers[m->L].n_tiles, (N + TILE - 1) / TILE, s);
  }
  m->profiling = was_profiling;
  if (rc != MADE_OK) return rc;
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

extern "C" int made_layer_activations(made_model* m, const uint8_t* x, int32_t N, int32_t layer, float* out,
                                      void* stream) {
  if (!m) return fail(MADE_ERR_ARG, "made_layer_activations: model is NULL");
  if (m->real) return fail(MADE_ERR_ARG, "made_layer_activations: the model has real states");
  if (N < 0 || N > (1 << 22)) return fail(MADE_ERR_ARG, "made_layer_activations: N=%d out of range [0, 2^22]", N);
  const int n_act = m->arch == 1 ? m->conv.n_conv : m->L;
  if (layer < 0 || layer >= n_act)
    return fail(MADE_ERR_ARG, "made_layer_activations: layer=%d, the model has %d layers with activations", layer, n_act);
  if (N > 0 && !out) return fail(MADE_ERR_ARG, "made_layer_activations: out is NULL");
  if (!x && m->arch != 1)
    return fail(MADE_ERR_ARG, "made_layer_activations: x is NULL (only the convolutional model keeps its activations)");
  HIP_TRY(hipSetDevice(m->device));
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  const bool was_profiling = m->profiling;
  m->profiling = false;
  TRY(settle(m, s));
  if (!x && N > m->ws.N_cap)
    return fail(MADE_ERR_ARG, "made_layer_activations: no call on %d or more images has run on this model yet", N);
  TRY(ensure_workspace(m, N, false));
  const void* act = nullptr;
  int rows = 0, width = 0, k_chunks = 0;
  const int* slot_unit = nullptr;
  if (m->arch == 1) {
    ConvNet& cv = m->conv;
    if (x) {
      const void* last = nullptr;
      launch_conv_trunk(m, x, N, nullptr, cv.H - 1, s, &last);
    }
    act = cv.act[layer];
    rows = N * cv.H * 32;
    width = cv.F;
    k_chunks = cv.F / chunk_elems(m);
  } else {
    TRY(launch_init_state(m, x, nullptr, N, s));
    RowSet rs{nullptr, nullptr, N, x};
    TRY(run_hidden(m, rs, nullptr, -1, s));
    act = m->ws.act[layer];
    rows = N;
    width = m->layers[layer].out_dim;
    k_chunks = m->layers[layer + 1].k_chunks;
    slot_unit = m->layers[layer].slot_unit;
  }
  m->profiling = was_profiling;
  const size_t total = (size_t)rows * width;
  const int blocks = (int)std::min<size_t>((total + 255) / 256, 16384);
  if (m->dtype == MADE_BF16)
    hipLaunchKernelGGL(unpack_activations_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)act, k_chunks,
                       slot_unit, rows, width, out);
  else
    hipLaunchKernelGGL(unpack_activations_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)act, k_chunks,
                       slot_unit, rows, width, out);
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

// One block of a call's schedule: positions [a, b) are iterated at most `cap` times (Algorithm 1: a single
// block [0, D); Algorithm 3: consecutive blocks; sequential sampling: D blocks of one position and one pass).
struct Block {
  int a = 0, b = 0, cap = 0;
  bool stop_test = true;          // false: no retire step (a one-pass block needs no stop test)
  bool whole_network = false;     // evaluate every output tile even though only [a, b) is re-drawn
  bool limited = false;           // evaluate only hidden units of degree < b (1-based), see run_hidden
  std::vector<int> hidden_limit;  // [L] when limited
  std::vector<int> hidden_frozen; // [L] when limited: units of degree <= a, whose inputs are positions before
                                  // the block: final, so their activations stay valid after the block's first pass
  int in_limit = -1, out_k_limit = -1;
  std::vector<int> k_first;       // [L + 1] when limited: the inputs of layer l before k_first[l] (chunk-rounded) are
                                  // frozen in this block: positions before a, resp. units of degree <= a
};

static Block make_block(const made_model* m, int a, int b, int cap, bool limited) {
  Block blk;
  blk.a = a;
  blk.b = b;
  blk.cap = cap;
  blk.limited = limited && m->arch == 0;
  if (blk.limited) {
    // positions <= b (1-based) read last-layer units of degree < b; those read units of degree <= their own,
    // and inputs of index <= b - 1
    blk.hidden_limit.resize(m->L);
    for (int l = 0; l < m->L; ++l) blk.hidden_limit[l] = m->cnt_lt[l][b];
    blk.hidden_frozen.resize(m->L);
    for (int l = 0; l < m->L; ++l) blk.hidden_frozen[l] = m->cnt_lt[l][std::min(a + 1, m->D)];
    blk.in_limit = b - 1;
    blk.out_k_limit = blk.hidden_limit[m->L - 1];
    const int kc = chunk_elems(m);
    blk.k_first.resize(m->L + 1);
    blk.k_first[0] = m->onehot ? 0 : a / kc * kc;      // (a one-hot first layer is a gather, not a product)
    for (int l = 1; l <= m->L; ++l) blk.k_first[l] = blk.hidden_frozen[l - 1] / kc * kc;
  }
  return blk;
}

// The sums over a block's frozen inputs, for every layer and every unit that later passes of the block still
// evaluate: P_l[sample, unit] = sum over the inputs i < k_first[l] of W_l[unit, i] * h_{l-1}[sample, i], from the
// activations the block's first pass has left (frozen units are final after it).  Plain launches of the layer
// kernels with the fp32 epilogue, K cut off at k_first[l], no bias, into one [n_pad, out_pad] buffer per layer.
static int fill_partial_sums(made_model* m, const RowSet& rs, const Block& blk, hipStream_t s) {
  Workspace& w = m->ws;
  if ((int)w.partial.size() != m->L + 1 || w.partial_cap < w.n_pad) {
    if (w.pending) {                                   // (queued kernels of an earlier call may still read the old buffers)
      HIP_TRY(hipDeviceSynchronize());
      w.pending = false;
    }
    for (float* p : w.partial)
      if (p) (void)hipFree(p);
    w.partial.assign(m->L + 1, nullptr);
    int widest = 0;
    for (int l = 0; l <= m->L; ++l) {
      HIP_TRY(hipMalloc((void**)&w.partial[l], (size_t)w.n_pad * m->layers[l].out_pad * sizeof(float)));
      widest = std::max(widest, m->layers[l].out_pad);
    }
    if (!w.zero_bias) {
      HIP_TRY(hipMalloc((void**)&w.zero_bias, (size_t)widest * sizeof(float)));
      HIP_TRY(hipMemset(w.zero_bias, 0, (size_t)widest * sizeof(float)));
    }
    w.partial_cap = w.n_pad;
  }
  const int row_tiles = (rs.n_rows + TILE - 1) / TILE;
  for (int l = 0; l <= m->L; ++l) {
    if (blk.k_first[l] <= 0) continue;
    const Layer& ly = m->layers[l];
    LayerArgs a = base_args(m, l, l == 0 ? w.enc : w.act[l - 1], rs);
    a.bias = w.zero_bias;
    a.k_cap = std::min(ly.in_pad, blk.k_first[l]);
    a.out = w.partial[l];
    a.ldo = ly.out_pad;
    a.n_cols = ly.out_pad;
    int tile_lo, tile_hi;
    if (l < m->L) {
      tile_hi = std::min(ly.n_tiles, (blk.hidden_limit[l] + TILE - 1) / TILE);
      tile_lo = std::min(tile_hi, blk.hidden_frozen[l] / TILE);
    } else {
      tile_lo = (blk.a * m->C) / TILE;
      tile_hi = (blk.b * m->C + TILE - 1) / TILE;
    }
    a.tile_begin = tile_lo;
    if (tile_hi - tile_lo <= 0) continue;
    launch_layer<EPI_LOGITS>(m, l, a, tile_hi - tile_lo, row_tiles, s);
    m->stats[2]++;
  }
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

// Enqueue the next pass of chain c's current block on the chain's stream.
static int enqueue_pass(made_model* m, Chain& c, const Block& blk, const float* noise, uint8_t* x,
                        bool flag_unconverged, bool force_tail = false) {
  Workspace& w = m->ws;
  hipStream_t s = c.stream;
  if (!c.block_started) {
    // the active list restarts as the chain's whole range (blocks without a stop test never shrink it)
    if (blk.stop_test || !c.iters_cleared) {
      const int padded = round_up(c.count, 2 * TILE);   // <= c.rows_cap
      // (the call's first reset also fills the second list with valid ids: a tile past the active count reads
      // list entries before it learns the count, and what an earlier, larger call left there would point
      // outside this call's buffers)
      hipLaunchKernelGGL(reset_rows_kernel, dim3((padded + 255) / 256), dim3(256), 0, s, c.rows[0],
                         c.iters_cleared ? nullptr : c.rows[1], c.n_rows[0], c.first, c.count, padded, w.changed,
                         c.iters_cleared ? nullptr : w.call_iters, c.done_ctr, c.done_ctr + FROZEN_WORDS);
      m->stats[2]++;
      c.iters_cleared = true;
    }
    c.block_started = true;
    c.bound = c.count;
  }
  c.bound_at_block_start = c.count;
  const int k = c.k_enq + 1;
  const int in = (k - 1) & 1, out = k & 1;
  // (grids, tile shapes and the place of the stop test are chosen for at most c.bound active samples: late passes
  // of a large batch run on a fraction of it)
  const int n_bound = std::max(1, std::min(c.bound, c.count));
  RowSet rs{c.rows[in], c.n_rows[in], n_bound, x, c.first};
  SampleIO io{noise, x, blk.a, blk.b, RetireArgs{}};
  // Tail-less stop test (see DeriveArgs): pass k only records which rows changed; pass k + 1's first kernel derives
  // its list from that, reports pass k's result and counts it.  The last allowed pass keeps the ordinary tail (no
  // pass follows it), and so does everything the conditions below exclude.
  const bool lazy_out = c.lazy && k < blk.cap && !force_tail;   // (force_tail: the last pass of a recorded call)
  const bool derive_in = c.lazy && k > 1;
  DeriveArgs dv;
  memset(&dv, 0, sizeof dv);
  if (derive_in) {
    // pass k - 1 read list (k - 2) & 1 and left its bits in set (k - 1) % 3; this pass's list goes where the
    // tail of pass k - 1 would have put it
    dv.enabled = 1;
    dv.rows_in = c.rows[k & 1];
    dv.n_in = c.n_rows[k & 1];
    dv.rows_out = c.rows[in];
    dv.n_out = c.n_rows[in];
    dv.mask_in = w.lazy_masks + ((k - 1) % 3) * DERIVE_WORDS;
    dv.mask_clear = w.lazy_masks + ((k + 1) % 3) * DERIVE_WORDS;
    dv.iters = w.call_iters;
    dv.pass = k - 1;
    dv.n_max = std::max(1, std::min(c.count, DERIVE_MAX_ROWS));
    dv.host_slot = c.d_pin + c.pin_base + ((int)c.log_first.size() - 1);
  }
  if (blk.stop_test) {
    const int slot = (int)c.log_first.size();
    if (slot >= c.pin_half - 1) return fail(MADE_ERR_HIP, "internal: pass log overflow");   // (the half's last word mirrors the flags)
    c.h_pin[c.pin_base + slot] = -1;
    io.retire.rows_in = c.rows[in];
    io.retire.n_in = c.n_rows[in];
    io.retire.rows_out = c.rows[out];
    io.retire.n_out = c.n_rows[out];
    io.retire.changed = w.changed;
    io.retire.iters = w.call_iters;
    io.retire.flags = w.flags;
    io.retire.done_ctr = c.done_ctr;
    io.retire.n_max = n_bound;
    io.retire.host_slot = c.d_pin + c.pin_base + slot;
    io.retire.host_flags = c.d_pin + c.pin_base + (c.pin_half - 1);
    io.retire.last_pass = (k == blk.cap);
    io.retire.flag_unconverged = flag_unconverged;
    io.retire.enabled = lazy_out ? 0 : 1;
    // Frozen positions (256-class output kernel): pass k starts at the position behind the lowest one pass k - 1
    // changed (word (k - 1) & 1; a block's first pass finds 0 there), records the lowest position it changes in word
    // 2 + (k & 1), and its tail turns that into the start of pass k + 1 and re-arms the other recording word.
    c.frozen = m->frozen_positions && m->arch == 0 && m->C == CAT_C && m->fused_categorical && !m->real &&
               n_bound < m->retire_split;
    if (c.frozen) {
      int* fw = c.done_ctr + FROZEN_WORDS;
      io.t_first_ptr = fw + ((k - 1) & 1);
      io.first_changed = fw + 2 + (k & 1);
      io.retire.fc_in = fw + 2 + (k & 1);
      io.retire.t_first_out = fw + (k & 1);
      io.retire.fc_reset = fw + 2 + ((k + 1) & 1);
      io.retire.host_t_first = c.d_pin + c.pin_len + c.pin_base + slot;
      c.h_pin[c.pin_len + c.pin_base + slot] = NO_CHANGE;
    }
    if (lazy_out) {
      io.lazy_mask = w.lazy_masks + (k % 3) * DERIVE_WORDS;
      m->stats[5]++;
    }
    c.log_first.push_back(k == 1);
  } else {
    rs = RowSet{c.rows[0], nullptr, c.count, x, c.first};   // no stop test: every sample of the chain takes the pass
  }
  if (m->arch == 1) {
    TRY(run_conv_pass(m, c.count, io, k == 1, blk.whole_network, s));
  } else {
    // (after a block's first pass the frozen prefix of every hidden layer is reused, not recomputed)
    const bool by_pos = hidden_by_position(m, rs, blk.limited);
    // Partial-sum cache (GS-Jacobi on long lists): from a block's second pass on, a layer multiplies only the inputs
    // that can still change and adds the sum over the frozen ones, which the block's second pass computes once
    // (from the activations its first pass left) for the units that are still evaluated.
    const bool cached = blk.limited && k > 1 && m->prefix_cache;
    const bool use_partial = cached && m->prefix_cache == 2 && m->C == 1 && !m->real &&
                             c.bound_at_block_start >= m->partial_batch && blk.cap > 2;
    PartialSums ps{blk.k_first.data(), w.partial.data()};
    if (use_partial && k == 2) TRY(fill_partial_sums(m, rs, blk, s));
    TRY(run_hidden(m, rs, blk.limited ? blk.hidden_limit.data() : nullptr, blk.in_limit, s,
                   cached ? blk.hidden_frozen.data() : nullptr, by_pos, nullptr, use_partial ? &ps : nullptr,
                   derive_in ? &dv : nullptr, (k == 1 && c.block == 0 && c.first_hidden_ready) ? 1 : 0));
    // a long list is retired by a kernel of its own, spread over the chip, instead of by the output kernel's
    // last workgroup
    const RetireArgs retire = io.retire;
    const bool split_retire = retire.enabled && n_bound >= m->retire_split;
    if (split_retire) io.retire.enabled = 0;
    TRY(run_output_sample(m, rs, io, blk.whole_network, blk.out_k_limit, s, by_pos, use_partial ? &ps : nullptr));
    if (split_retire) {
      hipLaunchKernelGGL(retire_kernel, dim3((n_bound + RETIRE_WG_ROWS - 1) / RETIRE_WG_ROWS), dim3(256), 0, s, retire);
      HIP_TRY(hipGetLastError());
      m->stats[2]++;
    }
  }
  c.k_enq = k;
  return MADE_OK;
}

// The device has not reported a pass for 30 s.  Passes that write the caller's buffers and the model's scratch
// memory are still queued (on `s` and possibly on the chains' own streams), so the model is marked: later calls
// are refused, and made_free / any reallocation waits for the whole device before it frees what they use.
static int give_up_waiting(made_model* m, hipStream_t s) {
  m->ws.pending = true;
  m->ws.pending_stream = s;
  m->poisoned = true;
  return fail(MADE_ERR_HIP, "device did not report the stop test of a pass within 30 s; kernels of this call are "
                            "still queued: synchronise the device before reusing the call's buffers");
}

// Run the block list on every chain.  Each chain works through the blocks on its own stream; the host keeps
// at most two unconfirmed passes per chain in flight (a pass enqueued after its chain emptied finds zero
// active rows and does nothing), and moves a chain to its next block as soon as the block's pass limit is
// enqueued or the device reported the chain's block as unchanged.  Returns after the caller's stream has been
// made to wait for all chains and has been synchronised.
static int run_chains(made_model* m, const std::vector<Block>& blocks, const float* noise, const uint8_t* x_init,
                      uint8_t* x, int N, bool flag_unconverged, int32_t* iters_out, hipStream_t s) {
  Workspace& w = m->ws;
  // split the batch into chains of whole 32-sample tiles
  int want = std::max(1, std::min(m->n_chains, (N + TILE - 1) / TILE));
  if (m->arch == 1) want = 1;   // the convolutional trunk always runs the whole batch
  const int per = round_up((N + want - 1) / want, TILE);
  const int n_chains = (N + per - 1) / per;
  int total_passes = 0;
  for (const Block& b : blocks) total_passes += b.cap;
  for (int i = 0; i < n_chains; ++i) {
    TRY(ensure_chain(m, (size_t)i, per, 2 * (total_passes + 8)));
    Chain& c = w.chains[i];
    c.pin_half = c.pin_len / 2;
    c.pin_base = (int)(c.calls++ & 1u) * c.pin_half;
    c.first = i * per;
    c.count = std::min(per, N - c.first);
    c.block = 0;
    c.k_enq = c.k_conf = 0;
    c.bound = c.count;
    c.block_started = c.finished = c.iters_cleared = false;
    c.lazy = false;
    c.first_hidden_ready = false;
    c.log_first.clear();
    c.stream = n_chains == 1 ? s : c.own_stream;   // a single chain needs no fork and join
  }
  w.call_iters = iters_out ? iters_out : w.iters;
  for (int i = 0; i < n_chains; ++i) w.chains[i].h_pin[w.chains[i].pin_base + w.chains[i].pin_half - 1] = 0;
  CallGraph* cg = nullptr;   // the recorded form of this call, if it has one
  if (n_chains == 1 && m->arch == 0) {
    // one chain on the caller's stream: the kernel that sets up the iterate also resets the chain's list and counters
    Chain& c = w.chains[0];
    CallReset r;
    memset(&r, 0, sizeof r);
    r.enabled = 1;
    r.rows = c.rows[0];
    r.rows_other = c.rows[1];
    r.n_rows = c.n_rows[0];
    r.first = c.first;
    r.count = c.count;
    r.padded = round_up(c.count, 2 * TILE);
    r.changed = w.changed;
    r.iters = w.call_iters;
    r.done_ctr = c.done_ctr;
    r.flags = w.flags;
    // (conditions of the tail-less stop test: Algorithm 1 of a Bernoulli MLP on one chain whose list fits one
    // workgroup's threads and whose layers run on the 32 x 32 tile kernel)
    c.lazy = m->lazy_retire && m->C == 1 && !m->real && blocks.size() == 1 && blocks[0].stop_test && !blocks[0].limited &&
             c.count <= DERIVE_MAX_ROWS && c.count < std::min(m->mid_batch, m->big_batch) && c.count < m->retire_split;
    r.lazy_masks = c.lazy ? w.lazy_masks : nullptr;
    r.frozen_words = c.done_ctr + FROZEN_WORDS;
    // Algorithm 1 of a Bernoulli MLP started from zeros: the first pass's first hidden layer multiplies a zero input,
    // so the set-up kernel writes its activations (ReLU of the bias, the same for every sample) and the pass starts at
    // the second hidden layer: one launch less per call.
    // (On the batches the large tile kernels serve, writing the activations costs what the layer costs: batch 32768,
    // 131 MB of scattered 8-byte stores, 115 us against a ~100 us launch.  There the layer is launched.)
    if (m->zero_start_fill && !x_init && m->C == 1 && !m->real && !m->onehot && blocks.size() == 1 && !blocks[0].limited &&
        blocks[0].stop_test && c.count < std::min(m->mid_batch, m->big_batch)) {
      r.h0_bias = m->layers[0].bias;
      r.h0_out = w.act[0];
      r.h0_chunks = m->layers[1].k_chunks;
      r.h0_units = m->layers[0].n_tiles * TILE;
      c.first_hidden_ready = true;
    }
    // A call of the tail-less kind is short (cfg2: 18 launches of ~5 us each) and bound by what the host pays per
    // launch: on request it is recorded once and replayed as one graph launch (see CallGraph).  The first call with
    // a key runs launch by launch and tells how many passes to record.
    if (m->call_graph && c.lazy && !m->profiling && s != nullptr) {   // (the null stream cannot be captured)
      for (CallGraph& g : m->graphs)
        if (g.noise == noise && g.x_init == x_init && g.x == x && g.iters == w.call_iters && g.stream == s && g.N == N &&
            g.cap == blocks[0].cap && g.pin_base == c.pin_base && g.flag_unconverged == flag_unconverged)
          cg = &g;
      if (!cg) {
        if ((int)m->graphs.size() >= CALL_GRAPHS_MAX) {
          size_t oldest = 0;
          for (size_t i = 1; i < m->graphs.size(); ++i)
            if (m->graphs[i].used < m->graphs[oldest].used) oldest = i;
          CallGraph& g = m->graphs[oldest];
          if (g.exec) {
            HIP_TRY(hipStreamSynchronize(g.stream));   // (it may still be executing)
            (void)hipGraphExecDestroy(g.exec);
            (void)hipGraphDestroy(g.graph);
          }
          m->graphs.erase(m->graphs.begin() + (long)oldest);
        }
        m->graphs.emplace_back();
        cg = &m->graphs.back();
        cg->noise = noise; cg->x_init = x_init; cg->x = x; cg->iters = w.call_iters; cg->stream = s; cg->N = N;
        cg->cap = blocks[0].cap; cg->pin_base = c.pin_base; cg->flag_unconverged = flag_unconverged;
      }
      cg->used = ++m->graph_clock;
      if (cg->exec && cg->needed > cg->passes && cg->passes < cg->cap) {   // the last call ran out of recorded passes
        HIP_TRY(hipStreamSynchronize(s));
        (void)hipGraphExecDestroy(cg->exec);
        (void)hipGraphDestroy(cg->graph);
        cg->exec = nullptr;
        cg->graph = nullptr;
      }
    }
    if (cg && cg->exec) {
      // replay: the host's bookkeeping of the recorded launches, then the launches themselves
      for (int slot = 0; slot < cg->passes; ++slot) c.h_pin[c.pin_base + slot] = -1;
      c.log_first = cg->log_first;
      c.k_enq = cg->passes;
      m->stats[2] += cg->kernels;
      m->stats[5] += cg->tail_less;
      HIP_TRY(hipGraphLaunch(cg->exec, s));
      c.block_started = true;
      c.iters_cleared = true;
      c.lazy = false;   // (the graph's last pass kept the tail: passes behind it are ordinary ones)
    } else if (cg && cg->needed > 0) {
      const int n_rec = std::min(cg->cap, std::max(2, cg->needed));
      const int64_t kernels0 = m->stats[2], tail_less0 = m->stats[5];
      HIP_TRY(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
      int rc = launch_init_state(m, x_init, x, N, s, &r);
      c.block_started = true;
      c.iters_cleared = true;
      for (int k = 1; rc == MADE_OK && k <= n_rec; ++k)
        rc = enqueue_pass(m, c, blocks[0], noise, x, flag_unconverged, k == n_rec);
      hipGraph_t graph = nullptr;
      const hipError_t end = hipStreamEndCapture(s, &graph);
      if (rc != MADE_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
      }
      HIP_TRY(end);
      hipGraphExec_t exec = nullptr;
      const hipError_t inst = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
      if (inst != hipSuccess) {
        (void)hipGraphDestroy(graph);
        HIP_TRY(inst);
      }
      cg->graph = graph;
      cg->exec = exec;
      cg->passes = n_rec;
      cg->log_first = c.log_first;
      cg->kernels = m->stats[2] - kernels0;
      cg->tail_less = m->stats[5] - tail_less0;
      HIP_TRY(hipGraphLaunch(cg->exec, s));
      c.lazy = false;
    } else {
      TRY(launch_init_state(m, x_init, x, N, s, &r));
      c.block_started = true;
      c.iters_cleared = true;
    }
  } else {
    TRY(launch_init_state(m, x_init, x, N, s));
    HIP_TRY(hipMemsetAsync(w.flags, 0, sizeof(int), s));
  }
  if (n_chains > 1) {
    HIP_TRY(hipEventRecord(w.fork_ev, s));
    for (int i = 0; i < n_chains; ++i) HIP_TRY(hipStreamWaitEvent(w.chains[i].stream, w.fork_ev, 0));
  }

  int n_finished = 0;
  auto last_progress = std::chrono::steady_clock::now();
  uint64_t spins = 0;
  while (n_finished < n_chains) {
    bool progressed = false;
    for (int i = 0; i < n_chains; ++i) {
      Chain& c = w.chains[i];
      if (c.finished) continue;
      const Block& blk = blocks[c.block];
      bool block_done = false;
      if (c.k_enq < blk.cap && c.k_enq - c.k_conf <= 1) {
        TRY(enqueue_pass(m, c, blk, noise, x, flag_unconverged));
        progressed = true;
      }
      if (!blk.stop_test) {
        c.k_conf = c.k_enq;
        block_done = c.k_enq == blk.cap;
      } else {
        // look (without blocking) at the oldest unconfirmed pass of this block
        if (c.k_conf < c.k_enq) {
          const int slot = (int)c.log_first.size() - (c.k_enq - c.k_conf);
          const int left = c.h_pin[c.pin_base + slot];
          if (left >= 0) {
            c.k_conf++;
            c.bound = std::min(c.bound, left);
            progressed = true;
            if (left == 0) block_done = true;
          }
        }
        if (c.k_enq == blk.cap) block_done = true;   // nothing more may be enqueued for this block
      }
      if (block_done) {
        if (cg) cg->needed = c.k_conf < c.k_enq && c.k_enq == blk.cap ? blk.cap : c.k_conf;
        c.block++;
        c.k_enq = c.k_conf = 0;
        c.block_started = false;
        if (c.block == blocks.size()) {
          c.finished = true;
          n_finished++;
          if (n_chains > 1) {
            HIP_TRY(hipEventRecord(c.done_ev, c.stream));
            HIP_TRY(hipStreamWaitEvent(s, c.done_ev, 0));
          }
        }
        progressed = true;
      }
    }
    if (progressed) {
      last_progress = std::chrono::steady_clock::now();
    } else if ((++spins & 0xfff) == 0 &&
               std::chrono::duration<double>(std::chrono::steady_clock::now() - last_progress).count() > 30.0) {
      return give_up_waiting(m, s);
    }
  }
  // Pass counts went straight to iters_out and the flags come through the chains' pinned words, so nothing is
  // copied back.  The call does not wait for the stream to drain either: it returns once the device has reported
  // every pass whose result matters.  What may still be queued are passes enqueued speculatively behind the one
  // that left no sample active: they find an empty list, touch nothing but the model's scratch memory, and are
  // ordered before whatever the caller enqueues next on this stream.
  const bool must_sync = m->arch == 1 || m->profiling;
  if (m->arch == 1)
    HIP_TRY(hipMemcpyAsync((void*)&w.h_pin[2], m->conv.rows_stat, sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
  if (must_sync) {
    HIP_TRY(hipStreamSynchronize(s));
    w.pending = false;
    m->stats[3]++;
  } else {
    const auto t0 = std::chrono::steady_clock::now();
    for (int i = 0; i < n_chains; ++i) {
      const Chain& c = w.chains[i];
      bool drained = false;             // a pass of this block has reported an empty list
      for (size_t j = 0; j < c.log_first.size(); ++j) {
        if (c.log_first[j]) drained = false;
        if (drained) continue;
        uint64_t polls = 0;
        while (c.h_pin[c.pin_base + j] < 0) {
          if ((++polls & 0xfff) == 0 &&
              std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > 30.0)
            return give_up_waiting(m, s);
        }
        if (c.h_pin[c.pin_base + j] == 0) drained = true;
      }
    }
    w.pending = true;
    w.pending_stream = s;
  }
  int call_flags = 0;
  for (int i = 0; i < n_chains; ++i) call_flags |= w.chains[i].h_pin[w.chains[i].pin_base + w.chains[i].pin_half - 1];
  if (m->arch == 1) {
    unsigned long long rows = 0;
    memcpy(&rows, (const void*)&w.h_pin[2], sizeof rows);
    m->stats[4] = (int64_t)rows;
  }
  prof_collect(m);
  // statistics from the chains' pass logs
  for (int i = 0; i < n_chains; ++i) {
    const Chain& c = w.chains[i];
    int64_t passes = 0;
    int active_in = 0;
    for (size_t j = 0; j < c.log_first.size(); ++j) {
      if (c.log_first[j]) active_in = c.count;
      if (active_in > 0) {
        passes++;
        m->stats[1] += active_in;
      }
      // visible output-layer weights this pass multiplied (Algorithm 1 of a 256-class model: the pass starts at the
      // position its predecessor's tail reported)
      if (active_in > 0 && m->arch == 0 && m->C == CAT_C && blocks.size() == 1 && blocks[0].stop_test) {
        int t_first = 0;
        if (c.frozen && !c.log_first[j]) {
          const int reported = c.h_pin[c.pin_len + c.pin_base + j - 1];
          t_first = std::min(m->D, std::max(0, reported));
        }
        const std::vector<int>& below = m->cnt_lt[m->L - 1];
        for (int t = t_first; t < m->D; ++t) m->stats[6] += (int64_t)below[t + 1] * m->C;
        m->stats[7] += (int64_t)(m->D - t_first) * active_in;
      }
      active_in = std::max(0, (int)c.h_pin[c.pin_base + j]);   // (an unreported pass is one that found the list empty)
    }
    m->stats[0] = std::max(m->stats[0], passes);
  }
  if (call_flags & 1)
    return fail(MADE_ERR_NOT_CONVERGED, "samples were still changing after the last allowed pass");
  return MADE_OK;
}

extern "C" int sequential_sample(made_model* m, const float* noise, int32_t N, int32_t mode, uint8_t* x_out,
                                 void* stream) {
  TRY(check_call(m, noise, N, x_out, "sequential_sample"));
  if (mode != 0 && mode != 1) return fail(MADE_ERR_ARG, "sequential_sample: mode=%d must be 0 or 1", mode);
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  memset(m->stats, 0, sizeof m->stats);
  m->ev_layer.clear();
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, true));
  std::vector<Block> blocks;
  blocks.reserve(m->D);
  for (int p = 0; p < m->D; ++p) {  // p = 0-based position, its 1-based index is t = p + 1
    Block blk = make_block(m, p, p + 1, 1, mode == 1);
    blk.stop_test = false;
    blk.whole_network = (mode == 0);
    blocks.push_back(std::move(blk));
  }
  TRY(run_chains(m, blocks, noise, nullptr, x_out, N, false, nullptr, s));
  m->stats[0] = m->D;
  m->stats[1] = (int64_t)m->D * N;
  return MADE_OK;
}

// The whole call in one cooperative launch (see persistent_sampler_kernel).  Returns 1 in *done when the call
// was served this way, 0 when the caller must take the stream-ordered path.
static int run_persistent(made_model* m, const float* noise, int N, const uint8_t* x_init, uint8_t* x, int block,
                          int cap, bool flag_unconverged, int32_t* iters_out, hipStream_t s, bool* done) {
  *done = false;
  if (m->arch != 0 || m->real || !m->use_persistent || m->persist_grid <= 0 || N > PERSIST_MAX_N) return MADE_OK;
  if ((uintptr_t)x % 4 != 0) return MADE_OK;   // the kernel re-reads symbols through their aligned 32-bit words
  Workspace& w = m->ws;
  PersistArgs p;
  memset(&p, 0, sizeof p);
  for (int l = 0; l <= m->L; ++l) {
    const Layer& ly = m->layers[l];
    PersistLayer& pl = p.layer[l];
    pl.W = ly.W;
    pl.bias = ly.bias;
    pl.tile_kend = ly.tile_kend;
    pl.cnt_lt = ly.cnt_lt;
    pl.out = l < m->L ? w.act[l] : nullptr;
    pl.in_pad = ly.in_pad;
    pl.k_chunks = ly.k_chunks;
    pl.n_tiles = ly.n_tiles;
    pl.out_dim = ly.out_dim;
    pl.out_chunks = l < m->L ? m->layers[l + 1].k_chunks : 0;
  }
  p.L = m->L;
  p.enc = w.enc;
  p.enc_chunks = m->layers[0].k_chunks;
  p.noise = noise;
  p.x_init = x_init;
  p.x = x;
  p.N = N;
  p.D = m->D;
  p.block = block;
  p.cap = cap;
  p.flag_unconverged = flag_unconverged;
  p.changed = w.changed;
  p.n_pad = w.n_pad;
  p.iters = w.iters;
  p.flags = w.flags;
  p.bar = w.bar;
  p.stats = w.dev_stats;
  p.spin_limit = 1u << 22;
  HIP_TRY(hipMemsetAsync(w.bar, 0, sizeof(unsigned), s));
  HIP_TRY(hipMemsetAsync(w.flags, 0, sizeof(int), s));
  void* args[] = {&p};
  prof_mark(m, m->L + 1, false, s);
  hipError_t e = m->dtype == MADE_BF16
                     ? hipLaunchCooperativeKernel((const void*)persistent_sampler_kernel<bf16_t>, dim3(m->persist_grid),
                                                  dim3(NW * 64), args, 0, s)
                     : hipLaunchCooperativeKernel((const void*)persistent_sampler_kernel<float>, dim3(m->persist_grid),
                                                  dim3(NW * 64), args, 0, s);
  prof_mark(m, m->L + 1, true, s);
  if (e != hipSuccess) {   // not launchable as a co-resident grid on this device: take the other path from now on
    (void)hipGetLastError();
    m->persist_grid = 0;
    m->ev_layer.clear();
    HIP_TRY(hipStreamSynchronize(s));
    return MADE_OK;
  }
  m->stats[2] += 1;
  if (iters_out) HIP_TRY(hipMemcpyAsync(iters_out, w.iters, (size_t)N * sizeof(int), hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipMemcpyAsync((void*)&w.h_pin[0], w.flags, sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipMemcpyAsync((void*)&w.h_pin[2], w.dev_stats, 2 * sizeof(long long), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  m->stats[3] += 1;
  prof_collect(m);
  long long st[2];
  memcpy(st, (const void*)&w.h_pin[2], sizeof st);
  m->stats[0] = st[0];
  m->stats[1] = st[1];
  *done = true;
  const int flags = w.h_pin[0];
  if (flags & 2) return fail(MADE_ERR_HIP, "persistent kernel: grid barrier timed out (workgroups not co-resident?)");
  if (flags & 1) return fail(MADE_ERR_NOT_CONVERGED, "samples were still changing after the last allowed pass");
  return MADE_OK;
}

// The whole call in one launch, each XCD iterating its own share of the samples (see xcd_sampler_kernel).  *done = true
// when the call was served this way; when the kernel backs out (workgroups not on the expected XCD, or not
// co-resident) the path is switched off for this model and the caller takes the per-layer launches.
static int run_xcd(made_model* m, const float* noise, int N, const uint8_t* x_init, uint8_t* x, int block,
                   int cap, bool flag_unconverged, int32_t* iters_out, hipStream_t s, bool* done) {
  *done = false;
  if (m->arch != 0 || m->real || m->C != 1 || !m->use_xcd || m->xcd_grid <= 0) return MADE_OK;
  const int per = (N + XCDS - 1) / XCDS;
  if (per > XCD_MAX_ROWS) return MADE_OK;
  // Where it pays (use_xcd = 1), measured on MI355X against the per-layer launches: the short passes of GS-Jacobi
  // blocks up to 1024 samples (D = 784, 2 x 2000: 1.2 against 2.3 ms for blocks of 16 at batch 128, 2.3 against 3.4 ms
  // at 1024); whole-network Jacobi passes only while a layer is at most 32 unit tiles wide and the batch at most 512
  // (196 / 2 x 500: 0.075 against 0.098 ms; 784 / 2 x 2000: 0.124 against 0.105 ms -- there a phase of this kernel,
  // with its device-scope operand loads and its barrier, costs more than a launch).
  if (m->use_xcd == 1) {
    int widest = 0;
    for (int l = 0; l <= m->L; ++l) widest = std::max(widest, m->layers[l].n_tiles);
    const bool gs = block < m->D;
    if (gs ? N > 1024 : (N > 512 || widest > 32)) return MADE_OK;
  }
  Workspace& w = m->ws;
  PersistArgs p;
  memset(&p, 0, sizeof p);
  for (int l = 0; l <= m->L; ++l) {
    const Layer& ly = m->layers[l];
    PersistLayer& pl = p.layer[l];
    pl.W = ly.W;
    pl.bias = ly.bias;
    pl.tile_kend = ly.tile_kend;
    pl.cnt_lt = ly.cnt_lt;
    pl.out = l < m->L ? w.act[l] : nullptr;
    pl.in_pad = ly.in_pad;
    pl.k_chunks = ly.k_chunks;
    pl.n_tiles = ly.n_tiles;
    pl.out_dim = ly.out_dim;
    pl.out_chunks = l < m->L ? m->layers[l + 1].k_chunks : 0;
  }
  p.L = m->L;
  p.enc = w.enc;
  p.enc_chunks = m->layers[0].k_chunks;
  p.noise = noise;
  p.x_init = x_init;
  p.x = x;
  p.N = N;
  p.D = m->D;
  p.block = block;
  p.cap = cap;
  p.flag_unconverged = flag_unconverged;
  p.changed = w.changed;
  p.n_pad = w.n_pad;
  p.iters = iters_out ? iters_out : w.iters;
  p.flags = w.flags;
  p.bar = w.bar;
  p.stats = w.dev_stats;
  p.spin_limit = 1u << 20;
  p.reg_base = w.xcd_calls * (unsigned)(m->xcd_grid / XCDS);
  p.call_id = (int)(++w.xcd_calls);
  p.host_report = w.xcd_report_dev;
  // The device flags are only ever set when the kernel backs out (after which this path is switched off), but the
  // per-layer scheduler and the persistent kernel share the word: the stream-ordered clear costs one small memset.
  HIP_TRY(hipMemsetAsync(w.flags, 0, sizeof(int), s));
  prof_mark(m, m->L + 1, false, s);
  if (m->dtype == MADE_BF16)
    hipLaunchKernelGGL(xcd_sampler_kernel<bf16_t>, dim3(m->xcd_grid), dim3(NW * 64), 0, s, p);
  else
    hipLaunchKernelGGL(xcd_sampler_kernel<float>, dim3(m->xcd_grid), dim3(NW * 64), 0, s, p);
  prof_mark(m, m->L + 1, true, s);
  HIP_TRY(hipGetLastError());
  m->stats[2] += 1;
  // Every XCD's first workgroup reports into pinned memory once its share of the batch is done; the call returns
  // when all have (results stay ordered on the stream like those of any launch).
  const auto t0 = std::chrono::steady_clock::now();
  uint64_t polls = 0;
  bool backed_out = false;
  for (;;) {
    if (w.xcd_report[64] != 0) { backed_out = true; break; }
    int n_done = 0;
    for (int g = 0; g < XCDS; ++g) n_done += (w.xcd_report[g * 8 + 5] == p.call_id);
    if (n_done == XCDS) break;
    if ((++polls & 0xfff) == 0 && std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > 30.0)
      return give_up_waiting(m, s);
  }
  if (m->profiling || backed_out) {
    HIP_TRY(hipStreamSynchronize(s));
    m->stats[3] += 1;
    w.pending = false;
  } else {
    w.pending = true;                // (workgroups may still be leaving the kernel; they touch nothing any more)
    w.pending_stream = s;
  }
  prof_collect(m);
  if (backed_out || w.xcd_report[64] != 0) {     // results are incomplete: take the other path from now on
    const int flags = w.xcd_report[64];
    unsigned counters[2 * XCDS * XCD_LINE];
    memset(counters, 0, sizeof counters);
    (void)hipMemcpy(counters, w.bar, sizeof counters, hipMemcpyDeviceToHost);
    char detail[256];
    int off = 0;
    for (int g = 0; g < XCDS; ++g)
      off += snprintf(detail + off, sizeof detail - off, " %u", counters[(XCDS + g) * XCD_LINE] - p.reg_base);
    (void)fail(MADE_OK, "xcd_sampler_kernel backed out (flags %d: 4 = more workgroups on an XCD than expected, 2 = a "
                        "barrier's wait ran out; workgroups registered per XCD:%s; expected %d each); per-layer launches "
                        "serve this model from now on", flags, detail, m->xcd_grid / XCDS);
    m->xcd_grid = 0;
    m->stats[2] = 0;
    w.xcd_report[64] = 0;
    return MADE_OK;
  }
  int call_flags = 0;
  for (int g = 0; g < XCDS; ++g) {
    const volatile int* r = w.xcd_report + g * 8;
    const int64_t passes = ((int64_t)r[1] << 32) | (uint32_t)r[0], sp = ((int64_t)r[3] << 32) | (uint32_t)r[2];
    m->stats[0] = std::max<int64_t>(m->stats[0], passes);
    m->stats[1] += sp;
    call_flags |= r[4];
  }
  *done = true;
  if (call_flags & 1) return fail(MADE_ERR_NOT_CONVERGED, "samples were still changing after the last allowed pass");
  return MADE_OK;
}

// The whole call in one launch of the sample-resident kernel (see resident_sampler_kernel): one workgroup per 32
// samples.  Returns 1 in *done when the call was served this way.
static int run_resident(made_model* m, const float* noise, int N, const uint8_t* x_init, uint8_t* x, int block,
                        int cap, bool flag_unconverged, int32_t* iters_out, hipStream_t s, bool* done) {
  *done = false;
  if (m->arch != 0 || m->real || !m->use_resident || m->res_lds_bytes <= 0) return MADE_OK;
  // One compute unit streams every visible weight of a pass (measured ~70 GB/s), against all of them in the
  // per-layer launches, whose passes cost ~20 us in dependent launches at batch ~100: the short passes of
  // GS-Jacobi blocks are where the resident kernel pays (2x and more); whole-network Jacobi passes are at best
  // even (0.116 vs 0.113 ms on a 196 / 2 x 500 network, 0.146 vs 0.097 ms on 784 / 2 x 512).
  if (m->use_resident == 2 && block >= m->D) return MADE_OK;
  Workspace& w = m->ws;
  ResidentArgs p;
  memset(&p, 0, sizeof p);
  for (int l = 0; l <= m->L; ++l) {
    const Layer& ly = m->layers[l];
    ResidentLayer& pl = p.layer[l];
    pl.W = ly.W;
    pl.bias = ly.bias;
    pl.tile_kend = ly.tile_kend;
    pl.cnt_lt = ly.cnt_lt;
    pl.in_pad = ly.in_pad;
    pl.k_chunks = ly.k_chunks;
    pl.n_tiles = ly.n_tiles;
    pl.out_dim = ly.out_dim;
    pl.lds_out = m->res_lds_out[l];
    pl.lds_bias = m->res_lds_bias[l];
    pl.lds_kend = m->res_lds_kend[l];
    pl.lds_cnt = m->res_lds_cnt[l];
  }
  p.L = m->L;
  p.lds_enc = m->res_lds_enc;
  p.lds_clear = m->res_lds_clear;
  p.noise = noise;
  p.x_init = x_init;
  p.x = x;
  p.N = N;
  p.D = m->D;
  p.block = std::min(block, m->D);
  p.cap = cap;
  p.flag_unconverged = flag_unconverged;
  p.io_aligned = (m->D % 4 == 0) && ((uintptr_t)noise % 16 == 0);
  p.iters = iters_out ? iters_out : w.iters;
  p.ctr = m->res_ctr;
  p.host = (unsigned long long*)m->res_host;
  const int grid = (N + RES_ROWS - 1) / RES_ROWS;
  prof_mark(m, m->L + 1, false, s);
  if (m->dtype == MADE_BF16)
    hipLaunchKernelGGL(resident_sampler_kernel<bf16_t>, dim3(grid), dim3(RES_W * 64), (size_t)m->res_lds_bytes, s, p);
  else
    hipLaunchKernelGGL(resident_sampler_kernel<float>, dim3(grid), dim3(RES_W * 64), (size_t)m->res_lds_bytes, s, p);
  prof_mark(m, m->L + 1, true, s);
  HIP_TRY(hipGetLastError());
  m->stats[2] += 1;
  HIP_TRY(hipStreamSynchronize(s));
  m->stats[3] += 1;
  prof_collect(m);
  const unsigned long long flags = m->res_host[0];
  m->stats[0] = (int64_t)m->res_host[1];
  m->stats[1] = (int64_t)m->res_host[2];
  *done = true;
  if (flags & 1) return fail(MADE_ERR_NOT_CONVERGED, "samples were still changing after the last allowed pass");
  return MADE_OK;
}

extern "C" int jacobi_sample(made_model* m, const float* noise, int32_t N, const uint8_t* x_init, int32_t max_iters,
                             uint8_t* x_out, int32_t* iters_out, void* stream) {
  TRY(check_call(m, noise, N, x_out, "jacobi_sample"));
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  memset(m->stats, 0, sizeof m->stats);
  m->ev_layer.clear();
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, true));
  const int cap = (max_iters <= 0 || max_iters > m->D) ? m->D : max_iters;
  bool done = false;
  TRY(run_persistent(m, noise, N, x_init, x_out, m->D, cap, cap < m->D, iters_out, s, &done));
  if (done) return MADE_OK;
  if (N <= 256) TRY(run_xcd(m, noise, N, x_init, x_out, m->D, cap, cap < m->D, iters_out, s, &done));
  if (done) return MADE_OK;
  TRY(run_resident(m, noise, N, x_init, x_out, m->D, cap, cap < m->D, iters_out, s, &done));
  if (done) return MADE_OK;
  if (N > 256) TRY(run_xcd(m, noise, N, x_init, x_out, m->D, cap, cap < m->D, iters_out, s, &done));
  if (done) return MADE_OK;
  std::vector<Block> blocks(1, make_block(m, 0, m->D, cap, false));
  return run_chains(m, blocks, noise, x_init, x_out, N, cap < m->D, iters_out, s);
}

extern "C" int gs_jacobi_sample(made_model* m, const float* noise, int32_t N, const uint8_t* x_init, int32_t block,
                                uint8_t* x_out, int32_t* iters_out, void* stream) {
  TRY(check_call(m, noise, N, x_out, "gs_jacobi_sample"));
  if (block < 1) return fail(MADE_ERR_ARG, "gs_jacobi_sample: block=%d must be >= 1", block);
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  memset(m->stats, 0, sizeof m->stats);
  m->ev_layer.clear();
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, true));
  bool done = false;
  TRY(run_persistent(m, noise, N, x_init, x_out, block, m->D, false, iters_out, s, &done));
  if (done) return MADE_OK;
  // (measured: the XCD-resident kernel is the faster of the two whole-call kernels up to ~256 samples, the
  // sample-resident one -- where the model fits it -- beyond)
  if (N <= 256) TRY(run_xcd(m, noise, N, x_init, x_out, block, m->D, false, iters_out, s, &done));
  if (done) return MADE_OK;
  TRY(run_resident(m, noise, N, x_init, x_out, block, m->D, false, iters_out, s, &done));
  if (done) return MADE_OK;
  if (N > 256) TRY(run_xcd(m, noise, N, x_init, x_out, block, m->D, false, iters_out, s, &done));
  if (done) return MADE_OK;
  std::vector<Block> blocks;
  for (int a = 0; a < m->D; a += block) {
    const int b = std::min(a + block, m->D);          // block = 0-based positions [a, b)
    blocks.push_back(make_block(m, a, b, b - a, true));
  }
  return run_chains(m, blocks, noise, x_init, x_out, N, false, iters_out, s);
}

// ------------------------------------------------------------------------------------------------
// entry points of models with real states (logistic conditionals); same schedulers as above, the symbol
// buffers are float [N, D] and a position counts as changed when it moved by more than eps
// ------------------------------------------------------------------------------------------------
extern "C" int made_forward_params(made_model* m, const float* x, int32_t N, float* params, void* stream) {
  TRY(check_call(m, x, N, params, "made_forward_params", true));
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  const bool was_profiling = m->profiling;
  m->profiling = false;
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, false));
  TRY(launch_init_state(m, (const uint8_t*)x, nullptr, N, s));
  RowSet rs{nullptr, nullptr, N};
  TRY(run_hidden(m, rs, nullptr, -1, s));
  LayerArgs a = base_args(m, m->L, m->ws.act[m->L - 1], rs);
  a.out = params;
  a.ldo = m->D * m->C;
  const int big_saved = m->big_batch, mid_saved = m->mid_batch;
  m->big_batch = m->mid_batch = 1 << 30;
  launch_layer<EPI_LOGITS>(m, m->L, a, m->layers[m->L].n_tiles, (N + TILE - 1) / TILE, s);
  m->big_batch = big_saved;
  m->mid_batch = mid_saved;
  m->profiling = was_profiling;
  HIP_TRY(hipGetLastError());
  return MADE_OK;
}

extern "C" int sequential_sample_real(made_model* m, const float* noise, int32_t N, int32_t mode, float* x_out,
                                      void* stream) {
  TRY(check_call(m, noise, N, x_out, "sequential_sample_real", true));
  if (mode != 0 && mode != 1) return fail(MADE_ERR_ARG, "sequential_sample_real: mode=%d must be 0 or 1", mode);
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  memset(m->stats, 0, sizeof m->stats);
  m->ev_layer.clear();
  m->call_eps = 0.f;
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, true));
  std::vector<Block> blocks;
  blocks.reserve(m->D);
  for (int p = 0; p < m->D; ++p) {
    Block blk = make_block(m, p, p + 1, 1, mode == 1);
    blk.stop_test = false;
    blk.whole_network = (mode == 0);
    blocks.push_back(std::move(blk));
  }
  TRY(run_chains(m, blocks, noise, nullptr, (uint8_t*)x_out, N, false, nullptr, s));
  m->stats[0] = m->D;
  m->stats[1] = (int64_t)m->D * N;
  return MADE_OK;
}

extern "C" int jacobi_sample_real(made_model* m, const float* noise, int32_t N, const float* x_init, float eps,
                                  int32_t max_iters, float* x_out, int32_t* iters_out, void* stream) {
  TRY(check_call(m, noise, N, x_out, "jacobi_sample_real", true));
  if (!(eps >= 0.f)) return fail(MADE_ERR_ARG, "jacobi_sample_real: eps must be >= 0");
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  memset(m->stats, 0, sizeof m->stats);
  m->ev_layer.clear();
  m->call_eps = eps;
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, true));
  const int cap = (max_iters <= 0 || max_iters > m->D) ? m->D : max_iters;
  std::vector<Block> blocks(1, make_block(m, 0, m->D, cap, false));
  return run_chains(m, blocks, noise, (const uint8_t*)x_init, (uint8_t*)x_out, N, cap < m->D, iters_out, s);
}

extern "C" int gs_jacobi_sample_real(made_model* m, const float* noise, int32_t N, const float* x_init, int32_t block,
                                     float eps, float* x_out, int32_t* iters_out, void* stream) {
  TRY(check_call(m, noise, N, x_out, "gs_jacobi_sample_real", true));
  if (block < 1) return fail(MADE_ERR_ARG, "gs_jacobi_sample_real: block=%d must be >= 1", block);
  if (!(eps >= 0.f)) return fail(MADE_ERR_ARG, "gs_jacobi_sample_real: eps must be >= 0");
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  memset(m->stats, 0, sizeof m->stats);
  m->ev_layer.clear();
  m->call_eps = eps;
  TRY(settle(m, s));
  TRY(ensure_workspace(m, N, true));
  std::vector<Block> blocks;
  for (int a = 0; a < m->D; a += block) {
    const int b = std::min(a + block, m->D);
    blocks.push_back(make_block(m, a, b, b - a, true));
  }
  return run_chains(m, blocks, noise, (const uint8_t*)x_init, (uint8_t*)x_out, N, false, iters_out, s);
}

template <typename P>
static int grow(P** p, size_t* cap, size_t need_bytes) {
  if (need_bytes <= *cap) return MADE_OK;
  if (*p) (void)hipFree(*p);
  *p = nullptr;
  *cap = 0;
  HIP_TRY(hipMalloc((void**)p, need_bytes));
  *cap = need_bytes;
  return MADE_OK;
}

// Algorithm 2 on the convolutional model.  Block i gets a copy of every image of its own ("virtual image" i * N + n,
// with its own symbols and its own per-layer activations), because inside an iteration the blocks' mixed state
// vectors differ: copy i holds the previous iterate everywhere except in block i, where the new states appear one
// by one.  An iteration: (1) all copies' symbols = previous iterate; one evaluation of the N real images, whose
// activations are then copied to every block's copies (rows above a block never change inside an iteration, so
// they are valid for all of them); (2) sub-steps q = 0 .. |block| - 1: every copy recomputes, in every layer, only
// the image rows between the state it drew last and the one it draws now, and the head draws that one state from
// the noise of the copy's real image; (3) the blocks' states are collected per real image, compared with the
// previous iterate (stop test) and become the new one.  One iteration costs |block| launches of the whole layer
// stack, each on about one row per block and image: with states that are expensive to evaluate this solver cannot
// compete with Algorithm 1 (which does the same work in one pass), it is here to complete the paper's family.
static int jacobi_gs_conv(made_model* m, const float* noise, int N, const uint8_t* x_init, int block, int max_iters,
                          uint8_t* x_out, int32_t* iters_out, hipStream_t s) {
  ConvNet& cv = m->conv;
  const int D = m->D;
  const int B = std::min(block, D);
  const int M = (D + B - 1) / B;
  const int64_t V64 = (int64_t)M * N;
  const size_t per_image = (size_t)cv.H * 32 * cv.F * elem_size(m);
  if (V64 > (1 << 20) || (double)V64 * per_image * cv.n_conv > 64e9)
    return fail(MADE_ERR_ARG, "jacobi_gs_sample: %d blocks x %d images = %lld copies of the image need more than 64 GB of "
                              "activations", M, N, (long long)V64);
  const int V = (int)V64;
  const int cap = (max_iters <= 0 || max_iters > M) ? M : max_iters;
  TRY(settle(m, s));
  TRY(ensure_workspace(m, V, false));
  Workspace& w = m->ws;
  TRY(grow(&m->jgs_xv, &m->jgs_xv_cap, (size_t)V * D));
  TRY(grow(&m->jgs_state, &m->jgs_state_cap, (size_t)(N + 1 + V) * sizeof(int)));
  int* state = m->jgs_state;
  int* n_active = m->jgs_state + N;
  int* state_one = m->jgs_state + N + 1;
  int* dirty_lo = cv.win;                  // [V]
  int* row_hi_of = cv.win + cv.win_pad;    // [V]
  HIP_TRY(hipMemsetAsync(state, 0, (size_t)(N + 1) * sizeof(int), s));
  HIP_TRY(hipMemsetAsync(w.flags, 0, sizeof(int), s));
  HIP_TRY(hipMemsetAsync(w.iters, 0, (size_t)N * sizeof(int), s));
  {
    const size_t total = (size_t)N * D;
    hipLaunchKernelGGL(copy_symbols_kernel, dim3((int)std::min<size_t>((total + 255) / 256, 4096)), dim3(256), 0, s, x_init,
                       x_out, total);
    m->stats[2]++;
  }
  ConvHeadArgs c;
  memset(&c, 0, sizeof c);
  c.W = cv.w_head;
  c.bias = cv.b_head;
  c.tile_kend = cv.head_tile_kend;
  c.noise = noise;
  c.x = m->jgs_xv;
  c.changed = w.changed;
  c.N = V;
  c.H = cv.H;
  c.state_lo = 0;
  c.state_hi = D;
  c.groups = std::max(1, std::min(V * cv.H, 85));
  c.state_one = state_one;
  c.noise_images = N;
  const size_t n16 = (size_t)N * per_image / 16;
  int k = 0;
  for (;;) {
    ++k;
    hipLaunchKernelGGL(jgs_conv_begin_kernel, dim3((int)std::min<size_t>(((size_t)V * D + 255) / 256, 8192)), dim3(256), 0, s,
                       x_out, m->jgs_xv, N, M, D);
    m->stats[2]++;
    const void* last = nullptr;
    launch_conv_trunk(m, m->jgs_xv, N, nullptr, cv.H - 1, s, &last);      // the previous iterate, every row
    if (M > 1)
      for (int l = 0; l < cv.n_conv; ++l) {
        hipLaunchKernelGGL(jgs_conv_broadcast_kernel, dim3((int)std::min<size_t>((n16 * (M - 1) + 255) / 256, 16384)), dim3(256),
                           0, s, (uint4*)cv.act[l], n16, M);
        m->stats[2]++;
      }
    for (int q = 0; q < B; ++q) {
      hipLaunchKernelGGL(jgs_conv_window_kernel, dim3((V + 255) / 256), dim3(256), 0, s, dirty_lo, row_hi_of, state_one, N, M,
                         D, B, q);
      m->stats[2]++;
      launch_conv_trunk(m, m->jgs_xv, V, dirty_lo, 0, s, &last, row_hi_of);
      c.A = last;
      launch_conv_head(m, c, s);
    }
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemsetAsync(n_active, 0, sizeof(int), s));
    hipLaunchKernelGGL(jgs_end_kernel, dim3(N), dim3(256), 0, s, x_out, m->jgs_xv, N, D, B, w.iters, state, k,
                       (k == cap) ? 1 : 0, (cap < M) ? 1 : 0, n_active, w.flags);
    m->stats[2]++;
    HIP_TRY(hipMemcpyAsync((void*)&w.h_pin[1], n_active, sizeof(int), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    m->stats[3]++;
    if (w.h_pin[1] == 0 || k == cap) break;
  }
  HIP_TRY(hipGetLastError());
  if (iters_out) HIP_TRY(hipMemcpyAsync(iters_out, w.iters, (size_t)N * sizeof(int), hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipMemcpyAsync((void*)&w.h_pin[0], w.flags, sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  prof_collect(m);
  m->stats[0] = k;
  m->stats[1] = (int64_t)k * B * V;
  if (w.h_pin[0] & 1)
    return fail(MADE_ERR_NOT_CONVERGED, "images were still changing after the last allowed iteration");
  return MADE_OK;
}

// Algorithm 2.  Every block keeps its own copy of the state vector ("virtual sample" (block i, sample n) =
// row i * np + n of a batch of M * np rows): it starts an iteration as the previous iterate and receives the
// block's new symbols one position at a time.  Sub-step q of an iteration evaluates the hidden layers on all
// virtual samples and then, in one launch, position a_i + q of every block i on that block's rows only.  After
// |block| sub-steps the blocks' positions are collected, compared with the previous iterate (per sample) and
// become the new iterate.
extern "C" int jacobi_gs_sample(made_model* m, const float* noise, int32_t N, const uint8_t* x_init, int32_t block,
                                int32_t max_iters, uint8_t* x_out, int32_t* iters_out, void* stream) {
  TRY(check_call(m, noise, N, x_out, "jacobi_gs_sample"));
  if (block < 1) return fail(MADE_ERR_ARG, "jacobi_gs_sample: block=%d must be >= 1", block);
  if (m->arch == 0 && m->C != 1)
    return fail(MADE_ERR_ARG, "jacobi_gs_sample: of the masked MLPs only those with Bernoulli positions are supported");
  if (N == 0) return MADE_OK;
  hipStream_t s = (hipStream_t)stream;
  memset(m->stats, 0, sizeof m->stats);
  m->ev_layer.clear();
  if (m->arch == 1) return jacobi_gs_conv(m, noise, N, x_init, block, max_iters, x_out, iters_out, s);
  const int D = m->D;
  const int B = std::min(block, D);
  const int M = (D + B - 1) / B;
  const int np = round_up(N, TILE);
  const int64_t V64 = (int64_t)M * np;
  if (V64 > (1 << 22))
    return fail(MADE_ERR_ARG, "jacobi_gs_sample: %d blocks x %d samples = %lld virtual samples exceed 2^22", M, np,
                (long long)V64);
  const int V = (int)V64;
  const int row_tiles = V / TILE, tiles_per_block = np / TILE;
  const int cap = (max_iters <= 0 || max_iters > M) ? M : max_iters;
  TRY(settle(m, s));
  TRY(ensure_workspace(m, V, false));
  Workspace& w = m->ws;
  TRY(grow(&m->jgs_xv, &m->jgs_xv_cap, (size_t)V * D));
  TRY(grow(&m->jgs_tab, &m->jgs_tab_cap, (size_t)B * row_tiles * sizeof(int)));
  TRY(grow(&m->jgs_state, &m->jgs_state_cap, (size_t)(N + 1) * sizeof(int)));
  {   // position drawn by row tile rt in sub-step q: a_i + q for its block i, or -1 past the block's end
    std::vector<int> tab((size_t)B * row_tiles);
    for (int q = 0; q < B; ++q)
      for (int rt = 0; rt < row_tiles; ++rt) {
        const int i = rt / tiles_per_block, pos = i * B + q;
        tab[(size_t)q * row_tiles + rt] = (pos < std::min((i + 1) * B, D)) ? pos : -1;
      }
    HIP_TRY(hipMemcpyAsync(m->jgs_tab, tab.data(), tab.size() * sizeof(int), hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));   // (tab is a local)
  }
  int* state = m->jgs_state;
  int* n_active = m->jgs_state + N;
  HIP_TRY(hipMemsetAsync(state, 0, (size_t)(N + 1) * sizeof(int), s));
  HIP_TRY(hipMemsetAsync(w.flags, 0, sizeof(int), s));
  HIP_TRY(hipMemsetAsync(w.iters, 0, (size_t)N * sizeof(int), s));
  {   // x_out = initial iterate
    const size_t total = (size_t)N * D;
    const int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(copy_symbols_kernel, dim3(blocks), dim3(256), 0, s, x_init, x_out, total);
    m->stats[2]++;
  }
  const RowSet rs{nullptr, nullptr, V};
  const int fill_blocks = (int)std::min<size_t>(((size_t)V * D + 255) / 256, 8192);
  int k = 0;
  for (;;) {
    ++k;
    if (m->dtype == MADE_BF16)
      hipLaunchKernelGGL((jgs_begin_kernel<bf16_t>), dim3(fill_blocks), dim3(256), 0, s, x_out, m->jgs_xv, (bf16_t*)w.enc,
                         m->layers[0].k_chunks, N, np, M, D);
    else
      hipLaunchKernelGGL((jgs_begin_kernel<float>), dim3(fill_blocks), dim3(256), 0, s, x_out, m->jgs_xv, (float*)w.enc,
                         m->layers[0].k_chunks, N, np, M, D);
    m->stats[2]++;
    for (int q = 0; q < B; ++q) {
      TRY(run_hidden(m, rs, nullptr, -1, s));
      LayerArgs a = base_args(m, m->L, w.act[m->L - 1], rs);
      a.noise = noise;
      a.x = m->jgs_xv;
      a.enc = w.enc;
      a.enc_chunks = m->layers[0].k_chunks;
      a.changed = w.changed;
      a.D = D;
      a.diag_pos = m->jgs_tab + (size_t)q * row_tiles;
      a.noise_mod = np;
      a.noise_n = N;
      a.n_launch_tiles = 1;
      a.row_tiles = row_tiles;
      prof_mark(m, m->L, false, s);
      if (m->dtype == MADE_BF16)
        hipLaunchKernelGGL((masked_layer_kernel<bf16_t, EPI_BERNOULLI>), dim3(row_tiles), dim3(NW * 64), 0, s, a);
      else
        hipLaunchKernelGGL((masked_layer_kernel<float, EPI_BERNOULLI>), dim3(row_tiles), dim3(NW * 64), 0, s, a);
      prof_mark(m, m->L, true, s);
      m->stats[2]++;
    }
    HIP_TRY(hipMemsetAsync(n_active, 0, sizeof(int), s));
    hipLaunchKernelGGL(jgs_end_kernel, dim3(N), dim3(256), 0, s, x_out, m->jgs_xv, np, D, B, w.iters, state, k,
                       (k == cap) ? 1 : 0, (cap < M) ? 1 : 0, n_active, w.flags);
    m->stats[2]++;
    HIP_TRY(hipMemcpyAsync((void*)&w.h_pin[1], n_active, sizeof(int), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    m->stats[3]++;
    if (w.h_pin[1] == 0 || k == cap) break;
  }
  HIP_TRY(hipGetLastError());
  if (iters_out) HIP_TRY(hipMemcpyAsync(iters_out, w.iters, (size_t)N * sizeof(int), hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipMemcpyAsync((void*)&w.h_pin[0], w.flags, sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  prof_collect(m);
  m->stats[0] = k;
  m->stats[1] = (int64_t)k * B * V;
  if (w.h_pin[0] & 1)
    return fail(MADE_ERR_NOT_CONVERGED, "samples were still changing after the last allowed iteration");
  return MADE_OK;
}

#ifdef JM_TRACE
#include "dev_trace_entry.hpp"   // development builds only: entry points that read the time stamps back
#endif

// ------------------------------------------------------------------------------------------------
// recurrent network: backward pass by Jacobi iteration
// ------------------------------------------------------------------------------------------------
#include "rnn_entry.hpp"
