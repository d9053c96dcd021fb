// Internal declarations shared by the host-side translation units of the library.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <map>
#include <string>
#include <vector>

#include "../../include/pmc.h"

namespace pmc {

// Records a message for pmc_last_error() and returns `code`.
int fail(int code, const char* fmt, ...);

// Tuning switches (tuning.cpp): -1 = the library decides.
enum Tuning { kTuneGemmTile, kTuneGemmGroup, kTuneGemmWgrad, kTuneAttnShape, kTuneWStreams, kTuneCount };
int tuning(Tuning t);

struct Schedule {
  int kind = -1;  // pmc_kind, or -1 for a custom V-shape block
  int d = 0, n = 0;
  bool grouped_bw = false;           // 1F1B: the stage is the unit of allocation
  bool fused = false;                // 1F1B, 1F1B-V: B and W of a chunk are one pass (nothing can be reordered,
                                     // and the chunk before waits for the end of the whole pass)
  std::vector<int32_t> block;        // [6][d]: rows F0, F1, B1, B0, W1, W0
  std::vector<pmc_pass> passes;      // all passes, global order
  std::vector<std::vector<pmc_pass>> per_device;
};

}  // namespace pmc

struct pmc_schedule {
  pmc::Schedule s;
};
