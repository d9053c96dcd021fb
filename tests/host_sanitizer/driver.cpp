// Drives the host-only part of the library (schedule construction, accounting, timing, reordering,
// adaptive search, tuning switches, error reporting) through the C ABI.  Built by
// tests/test_host_sanitizers.py with AddressSanitizer and UndefinedBehaviorSanitizer: any
// out-of-bounds access, leak, use after free, signed overflow or misaligned access in that code
// ends the run with a non-zero status.  No GPU code is linked.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/pmc.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "check failed at line %d: %s (%s)\n", __LINE__, #cond, pmc_last_error()); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

int main() {
  long passes_seen = 0;
  for (int kind = 0; kind <= 4; ++kind)
    for (int d = 1; d <= 9; ++d)
      for (int n : {1, 2, d, 3 * d + 1}) {
        pmc_schedule* s = nullptr;
        CHECK(pmc_schedule_build(kind, d, n, &s) == PMC_OK);
        CHECK(pmc_schedule_devices(s) == d && pmc_schedule_microbatches(s) == n);
        const int total = pmc_schedule_num_passes(s);
        CHECK(total == 6 * d * n);
        std::vector<int32_t> block(6 * d);
        CHECK(pmc_schedule_block(s, block.data(), (int32_t)block.size()) == PMC_OK);
        CHECK(pmc_schedule_block(s, block.data(), (int32_t)block.size() - 1) == PMC_ERR_INVALID);
        std::vector<pmc_pass> order(total);
        CHECK(pmc_schedule_global_order(s, order.data(), total) == PMC_OK);
        CHECK(pmc_schedule_global_order(s, order.data(), total - 1) == PMC_ERR_INVALID);
        for (int i = 0; i < d; ++i) CHECK(pmc_schedule_device_order(s, i, order.data(), 6 * n) == PMC_OK);
        CHECK(pmc_schedule_device_order(s, d, order.data(), 6 * n) == PMC_ERR_INVALID);
        std::vector<pmc_device_peak> peaks(d);
        CHECK(pmc_schedule_account(s, 1000, 7, peaks.data(), d) == PMC_OK);
        CHECK(pmc_schedule_account(s, 1000, 2000, peaks.data(), d) == PMC_ERR_INVALID);
        double span = 0.0;
        CHECK(pmc_schedule_makespan(s, 1.0, 1.25, 0.75, &span) == PMC_OK && span > 0.0);
        pmc_schedule* r = nullptr;
        CHECK(pmc_schedule_reorder(s, &r) == PMC_OK);
        double span_r = 0.0;
        CHECK(pmc_schedule_makespan(r, 1.0, 1.25, 0.75, &span_r) == PMC_OK && span_r <= span + 1e-9);
        CHECK(pmc_schedule_account(r, 1000, 7, peaks.data(), d) == PMC_OK);
        passes_seen += total;
        pmc_schedule_destroy(r);
        pmc_schedule_destroy(s);
      }
  // custom V-shape blocks, legal and colliding
  int legal = 0, illegal = 0;
  for (int a = 1; a <= 6; ++a)
    for (int b = 1; b <= 6; ++b)
      for (int c = 1; c <= 6; ++c) {
        pmc_schedule* s = nullptr;
        const int rc = pmc_schedule_build_vshape(5, 7, 4, 2, a, b, c, &s);
        CHECK(rc == PMC_OK || rc == PMC_ERR_ILLEGAL_BLOCK);
        if (rc == PMC_OK) {
          ++legal;
          pmc_schedule_destroy(s);
        } else {
          ++illegal;
        }
      }
  CHECK(legal > 0 && illegal > 0);
  // adaptive search, with and without reordering, feasible and infeasible limits
  for (int reorder = 0; reorder <= 1; ++reorder) {
    pmc_schedule* s = nullptr;
    pmc_search_result res;
    CHECK(pmc_schedule_search(3, 6, 4, 1.0, 1.1, 0.8, 2, reorder, &res, &s) == PMC_OK);
    CHECK(res.peak_units <= 4 && res.feasible > 0 && res.candidates >= res.feasible);
    pmc_schedule_destroy(s);
    s = nullptr;
    CHECK(pmc_schedule_search(3, 6, 1, 1.0, 1.0, 1.0, 2, reorder, nullptr, &s) == PMC_ERR_ILLEGAL_BLOCK);
  }
  // bad arguments
  pmc_schedule* s = nullptr;
  CHECK(pmc_schedule_build(9, 4, 4, &s) == PMC_ERR_INVALID);
  CHECK(pmc_schedule_build(PMC_VHALF, 0, 4, &s) == PMC_ERR_INVALID);
  CHECK(pmc_schedule_build(PMC_VHALF, 4, 4, nullptr) == PMC_ERR_INVALID);
  CHECK(pmc_schedule_reorder(nullptr, &s) == PMC_ERR_INVALID);
  CHECK(pmc_schedule_devices(nullptr) == 0);
  pmc_schedule_destroy(nullptr);
  // tuning switches
  int32_t v = 0;
  CHECK(pmc_tuning_set("gemm_tile", 3) == PMC_OK && pmc_tuning_get("gemm_tile", &v) == PMC_OK && v == 3);
  CHECK(pmc_tuning_set("gemm_tile", 9) == PMC_ERR_INVALID);
  CHECK(pmc_tuning_set("nope", 1) == PMC_ERR_INVALID && pmc_tuning_set(nullptr, 1) == PMC_ERR_INVALID);
  CHECK(pmc_tuning_get("gemm_tile", nullptr) == PMC_ERR_INVALID);
  CHECK(pmc_tuning_set("gemm_tile", -1) == PMC_OK);
  std::printf("host sanitizer driver: %ld passes generated, %d legal / %d colliding custom blocks\n", passes_seen, legal, illegal);
  return 0;
}
