// Internal entry points of the chunk/pool layer used by the schedule replayer.
#pragma once
#include <hip/hip_runtime.h>

#include "pmc_internal.h"

namespace pmc {
int chunk_reserve(pmc_chunk* ch, int32_t mb, int device);
int chunk_forward(pmc_chunk* ch, int32_t mb, const void* x, void* y, int device);
int chunk_backward_input(pmc_chunk* ch, int32_t mb, const void* dy, void* dx);
int chunk_backward_weight_one(pmc_chunk* ch, int32_t mb, bool release);
int chunk_release(pmc_chunk* ch, int32_t mb);
void chunk_release_all(pmc_chunk* ch);
size_t chunk_unit_bytes(const pmc_chunk* ch);
size_t chunk_stats_bytes(const pmc_chunk* ch);
size_t chunk_workspace_bytes(const pmc_chunk* ch);
pmc_ctx* chunk_ctx(const pmc_chunk* ch);
const pmc_chunk_cfg& chunk_cfg(const pmc_chunk* ch);
hipStream_t ctx_stream(const pmc_ctx* ctx);
char* ctx_workspace(const pmc_ctx* ctx, size_t* bytes);
void ctx_device_peaks(pmc_ctx* ctx, int d, int64_t unit_bytes, pmc_device_peak* out);
}  // namespace pmc
