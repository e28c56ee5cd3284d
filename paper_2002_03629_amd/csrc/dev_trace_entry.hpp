// Development builds only (-DJM_TRACE): read (and clear) the time stamps of dev_trace.hpp.  Not declared in the
// public headers and not part of the library that is shipped.
#pragma once
#ifdef JM_TRACE
extern "C" int jm_debug_read_trace(unsigned long long* out) {
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(jm::g_trace), sizeof(unsigned long long) * 64 * 256 * 5) != hipSuccess) return -1;
  static std::vector<unsigned long long> zeros(64 * 256 * 5, 0);
  (void)hipMemcpyToSymbol(HIP_SYMBOL(jm::g_trace), zeros.data(), sizeof(unsigned long long) * 64 * 256 * 5);
  return 0;
}
extern "C" int jm_debug_read_tile_trace(unsigned long long* out) {
  return hipMemcpyFromSymbol(out, HIP_SYMBOL(jm::g_tile_trace), sizeof(unsigned long long) * 1024 * 8) == hipSuccess ? 0 : -1;
}
#endif
