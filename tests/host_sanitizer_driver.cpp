// Host-code check under AddressSanitizer / UndefinedBehaviorSanitizer, no GPU involved (test code).
//
// The library's host side -- argument checks, masks, degree sort, packing of the weights into the fragment-major
// layout, the convolution's tap tables, clean-up after failures -- is run here against a stand-in for the HIP runtime
// that this program defines itself: "device" allocations are host allocations, copies are memcpy.  The sanitized
// library therefore runs made_init / made_conv_init / made_free to the end, and every upload is checked against the
// size of the buffer it goes to.  No kernel is launched.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <random>
#include <vector>

#include "jacobi_made.h"

static std::map<void*, size_t> g_live;   // stand-in device allocations

extern "C" {
hipError_t hipMalloc(void** p, size_t n) {
  *p = malloc(n ? n : 1);
  g_live[*p] = n;
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void* p) {
  if (!p) return hipSuccess;
  if (!g_live.erase(p)) { fprintf(stderr, "hipFree of a pointer that is not live\n"); abort(); }
  free(p);
  return hipSuccess;
}
hipError_t hipMemcpy(void* d, const void* s, size_t n, hipMemcpyKind) { memcpy(d, s, n); return hipSuccess; }
hipError_t hipMemset(void* d, int v, size_t n) { memset(d, v, n); return hipSuccess; }
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipDeviceSynchronize(void) { return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipGetSymbolAddress(void** p, const void*) { static char scratch[64]; *p = scratch; return hipSuccess; }
hipError_t hipHostMalloc(void** p, size_t n, unsigned) { *p = malloc(n ? n : 1); return hipSuccess; }
hipError_t hipHostFree(void* p) { free(p); return hipSuccess; }
hipError_t hipHostGetDevicePointer(void** d, void* h, unsigned) { *d = h; return hipSuccess; }
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) { *v = 256; return hipSuccess; }
hipError_t hipFuncSetAttribute(const void*, hipFuncAttribute, int) { return hipSuccess; }
hipError_t hipOccupancyMaxActiveBlocksPerMultiprocessor(int* n, const void*, int, size_t) { *n = 1; return hipSuccess; }
}

static int failures = 0;
#define EXPECT(cond)                                                          \
  do {                                                                        \
    if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static void mlp_case(int D, int C, std::vector<int> hidden, int dtype, int real, int onehot, unsigned seed) {
  std::mt19937 g(seed);
  std::uniform_int_distribution<int> deg(1, D - 1);
  std::normal_distribution<float> nrm(0.f, 1.f);
  const int L = (int)hidden.size();
  std::vector<std::vector<int32_t>> degrees(L);
  std::vector<const int32_t*> dp(L);
  for (int l = 0; l < L; ++l) {
    degrees[l].resize(hidden[l]);
    for (auto& v : degrees[l]) v = deg(g);
    dp[l] = degrees[l].data();
  }
  std::vector<std::vector<float>> W(L + 1), b(L + 1);
  std::vector<const float*> wp(L + 1), bp(L + 1);
  for (int l = 0; l <= L; ++l) {
    const size_t in = l == 0 ? (size_t)D * (onehot ? C : 1) : hidden[l - 1];
    const size_t out = l == L ? (size_t)D * C : hidden[l];
    W[l].resize(in * out);
    for (auto& v : W[l]) v = nrm(g) * 0.1f;
    b[l].resize(out);
    for (auto& v : b[l]) v = nrm(g);
    wp[l] = W[l].data();
    bp[l] = (l & 1) ? nullptr : b[l].data();   // (some biases NULL)
  }
  made_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.D = D;
  cfg.C = C;
  cfg.n_hidden = L;
  cfg.hidden = hidden.data();
  cfg.dtype = dtype;
  cfg.real = real;
  cfg.onehot = onehot;
  made_model* m = nullptr;
  const int rc = made_init(&cfg, dp.data(), wp.data(), bp.data(), &m);
  if (rc != MADE_OK) fprintf(stderr, "made_init(D=%d C=%d): %s\n", D, C, made_last_error());
  EXPECT(rc == MADE_OK && m != nullptr);
  if (m) {
    int64_t nnz[8] = {0};
    EXPECT(made_layer_nnz(m, nnz, L + 1) == MADE_OK && nnz[0] > 0);
    EXPECT(made_set_option(m, MADE_OPT_CHAINS, 3) == MADE_OK);
    EXPECT(made_set_option(m, MADE_OPT_CHAINS, 99) == MADE_ERR_ARG);
    EXPECT(made_set_option(m, 12345, 1) == MADE_ERR_ARG);
    int64_t st[8];
    EXPECT(made_last_stats(m, st, 8) == MADE_OK);
    // calls with bad arguments are refused before any device work
    EXPECT(jacobi_sample(m, nullptr, 4, nullptr, 0, nullptr, nullptr, nullptr) == MADE_ERR_ARG);
    EXPECT(gs_jacobi_sample(m, nullptr, 4, nullptr, 0, nullptr, nullptr, nullptr) == MADE_ERR_ARG);
    EXPECT(sequential_sample(m, nullptr, -1, 0, nullptr, nullptr) == MADE_ERR_ARG);
    EXPECT(made_free(m) == MADE_OK);
  }
}

static void conv_case(int H, int F, int k, int n_conv, int dtype, unsigned seed) {
  std::mt19937 g(seed);
  std::normal_distribution<float> nrm(0.f, 1.f);
  std::vector<std::vector<float>> W(n_conv + 1), b(n_conv + 1);
  std::vector<const float*> wp(n_conv + 1), bp(n_conv + 1);
  for (int l = 0; l <= n_conv; ++l) {
    const size_t out = l == n_conv ? 3 * 256 : F, in = l == 0 ? 3 : F, kk = l == n_conv ? 1 : (size_t)k * k;
    W[l].resize(out * kk * in);
    for (auto& v : W[l]) v = nrm(g) * 0.05f;
    b[l].resize(out);
    for (auto& v : b[l]) v = nrm(g);
    wp[l] = W[l].data();
    bp[l] = b[l].data();
  }
  made_conv_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.H = H;
  cfg.W = 32;
  cfg.C = 256;
  cfg.F = F;
  cfg.k = k;
  cfg.n_conv = n_conv;
  cfg.dtype = dtype;
  made_model* m = nullptr;
  const int rc = made_conv_init(&cfg, wp.data(), bp.data(), &m);
  if (rc != MADE_OK) fprintf(stderr, "made_conv_init(H=%d F=%d k=%d): %s\n", H, F, k, made_last_error());
  EXPECT(rc == MADE_OK && m != nullptr);
  if (m) EXPECT(made_free(m) == MADE_OK);
}

int main() {
  // argument errors
  made_model* m = nullptr;
  EXPECT(made_init(nullptr, nullptr, nullptr, nullptr, &m) == MADE_ERR_ARG);
  EXPECT(made_free(nullptr) == MADE_OK);
  EXPECT(strlen(made_last_error()) > 0);
  {
    made_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.D = 1;   // too few positions
    int32_t h = 4;
    cfg.hidden = &h;
    cfg.n_hidden = 1;
    cfg.C = 1;
    EXPECT(made_init(&cfg, nullptr, nullptr, nullptr, &m) == MADE_ERR_ARG);
  }
  // whole initialisations: ragged sizes, both dtypes, every kind of position
  mlp_case(64, 1, {256}, MADE_F32, 0, 0, 1);
  mlp_case(37, 1, {45, 71}, MADE_BF16, 0, 0, 2);
  mlp_case(196, 1, {500, 500}, MADE_BF16, 0, 0, 3);
  mlp_case(12, 256, {70, 33}, MADE_BF16, 0, 0, 4);
  mlp_case(9, 5, {40}, MADE_F32, 0, 0, 5);
  mlp_case(11, 256, {64, 48}, MADE_BF16, 0, 1, 6);
  mlp_case(23, 2, {60, 60}, MADE_F32, 1, 0, 7);
  conv_case(3, 64, 5, 3, MADE_BF16, 8);
  conv_case(2, 64, 3, 2, MADE_F32, 9);
  conv_case(4, 128, 5, 3, MADE_BF16, 10);
  conv_case(2, 128, 7, 2, MADE_BF16, 11);
  EXPECT(g_live.empty());   // made_free released every stand-in device allocation
  if (!g_live.empty()) fprintf(stderr, "%zu allocations still live\n", g_live.size());
  printf("host sanitizer driver: %d failures\n", failures);
  return failures ? 1 : 0;
}
