// Process-wide tuning switches (tests and kernel tuning): which GEMM tile shape, which attention
// launch family, how many streams the W pass uses.  Each switch is an atomic integer, -1 meaning
// "the library decides".  The environment (PMC_GEMM_TILE, PMC_GEMM_GROUP, PMC_GEMM_WGRAD,
// PMC_ATTN_SHAPE, PMC_W_STREAMS) is read ONCE, at the first use of any switch; afterwards only
// pmc_tuning_set changes a value, so the launch paths never touch the environment.
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "pmc_internal.h"

namespace pmc {
namespace {

struct Entry {
  const char* name;
  const char* env;
  int lo, hi;  // accepted range
};
constexpr Entry kEntries[kTuneCount] = {
    {"gemm_tile", "PMC_GEMM_TILE", 0, 4},      {"gemm_group", "PMC_GEMM_GROUP", 1, 64},
    {"gemm_wgrad", "PMC_GEMM_WGRAD", 0, 2},    {"attn_shape", "PMC_ATTN_SHAPE", 0, 2},
    {"w_streams", "PMC_W_STREAMS", 1, 2},
};
std::atomic<int> g_value[kTuneCount];
std::once_flag g_once;

void read_environment() {
  for (int i = 0; i < kTuneCount; ++i) {
    int v = -1;
    if (const char* s = std::getenv(kEntries[i].env)) {
      char* end = nullptr;
      const long parsed = std::strtol(s, &end, 10);
      if (end != s && *end == 0 && parsed >= kEntries[i].lo && parsed <= kEntries[i].hi) v = (int)parsed;
    }
    g_value[i].store(v, std::memory_order_relaxed);
  }
}

int find(const char* name) {
  if (!name) return -1;
  for (int i = 0; i < kTuneCount; ++i)
    if (std::strcmp(name, kEntries[i].name) == 0) return i;
  return -1;
}

}  // namespace

int tuning(Tuning t) {
  std::call_once(g_once, read_environment);
  return g_value[t].load(std::memory_order_relaxed);
}

}  // namespace pmc

using namespace pmc;

extern "C" {

int pmc_tuning_set(const char* name, int32_t value) {
  std::call_once(g_once, read_environment);
  const int i = find(name);
  if (i < 0) return fail(PMC_ERR_INVALID, "pmc_tuning_set: unknown switch '%s'", name ? name : "(null)");
  if (value != -1 && (value < kEntries[i].lo || value > kEntries[i].hi))
    return fail(PMC_ERR_INVALID, "pmc_tuning_set: %s takes -1 or %d..%d, got %d", name, kEntries[i].lo, kEntries[i].hi, value);
  g_value[i].store(value, std::memory_order_relaxed);
  return PMC_OK;
}

int pmc_tuning_get(const char* name, int32_t* value) {
  std::call_once(g_once, read_environment);
  const int i = find(name);
  if (i < 0 || !value) return fail(PMC_ERR_INVALID, "pmc_tuning_get: unknown switch or NULL result");
  *value = g_value[i].load(std::memory_order_relaxed);
  return PMC_OK;
}

}  // extern "C"
