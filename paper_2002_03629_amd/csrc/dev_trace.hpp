// Development instrumentation, compiled in only with -DJM_TRACE (never in the library that is shipped and
// benchmarked): workgroups write wall-clock time stamps into two device arrays that a debug entry point reads
// back.  Without JM_TRACE every hook below expands to nothing and the arrays do not exist.
#pragma once

#ifdef JM_TRACE
// (included from inside namespace jm)
__device__ unsigned long long g_tile_trace[1024 * 8];      // [workgroup][stamp 0..7]
__device__ unsigned long long g_trace[64 * 256 * 5];        // persistent kernel: [barrier][workgroup][stage 1..5]
#define JM_TSTAMP(i, drain)                                                           \
  do {                                                                                \
    if (drain) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");            \
    if (threadIdx.x == 0 && blockIdx.x < 1024) g_tile_trace[blockIdx.x * 8 + (i)] = wall_clock64(); \
  } while (0)
#define JM_TRACE_VALUE(i, v)                                                          \
  do {                                                                                \
    if (threadIdx.x == 0 && blockIdx.x < 1024) g_tile_trace[blockIdx.x * 8 + (i)] = (v); \
  } while (0)
// time a wave spends inside a wait (summed over a loop; reported next to a count in one trace word)
#define JM_WAIT_DECL() unsigned long long jm_wait_sum_ = 0, jm_wait_t0_ = 0
#define JM_WAIT_BEGIN() jm_wait_t0_ = wall_clock64()
#define JM_WAIT_END() jm_wait_sum_ += wall_clock64() - jm_wait_t0_
#define JM_WAIT_PACK(count) ((unsigned long long)(count) | (jm_wait_sum_ << 16))
#define JM_TRACE_TAIL_DONE()                                                          \
  do {                                                                                \
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                       \
    if (threadIdx.x == 0) g_tile_trace[1023 * 8] = wall_clock64();                    \
  } while (0)
// per workgroup and grid barrier: arrival / after the release fence / after the arrival atomic / after the wait /
// after the acquire fence
#define JM_STAMP(tag)                                                                            \
  do {                                                                                           \
    const unsigned b_ = epoch / gridDim.x - 1;                                                   \
    if (b_ < 64 && blockIdx.x < 256) g_trace[(b_ * 256 + blockIdx.x) * 5 + (tag)-1] = wall_clock64(); \
  } while (0)
// sample-resident kernel: wave JM_RES_TRACE_WAVE of workgroup 0 stamps the phases of its first 128 passes
#ifndef JM_RES_TRACE_WAVE
#define JM_RES_TRACE_WAVE 0
#endif
#define RES_STAMP(pass, i)                                                                              \
  do {                                                                                                  \
    if (blockIdx.x == 0 && threadIdx.x == JM_RES_TRACE_WAVE * 64 && (pass) < 128)                        \
      g_tile_trace[(pass) * 8 + (i)] = wall_clock64();                                                  \
  } while (0)
#else
#define RES_STAMP(pass, i) do { } while (0)
#define JM_TSTAMP(i, drain) do { } while (0)
#define JM_TRACE_VALUE(i, v) do { } while (0)
#define JM_WAIT_DECL() do { } while (0)
#define JM_WAIT_BEGIN() do { } while (0)
#define JM_WAIT_END() do { } while (0)
#define JM_WAIT_PACK(count) (count)
#define JM_TRACE_TAIL_DONE() do { } while (0)
#define JM_STAMP(tag) do { } while (0)
#endif
