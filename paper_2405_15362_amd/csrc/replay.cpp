// Single-GPU schedule replayer: runs every pass of a schedule's one-stream order on the context's
// stream.  The simulated devices share the GPU; what would be a send/recv between pipeline stages
// is a hand-over of a workspace buffer from the producing pass to the consuming one.  Activation
// lifetimes follow Section 2.2 of the paper: a chunk's unit is taken from the pool when its F
// starts and returned when its W has ended (for 1F1B the stage takes both chunks' units when its
// F starts and returns both when its fused backward ends), and each unit is charged to the
// simulated device that owns the chunk, so the pool's per-device high-water marks are the
// schedule's peak activation memory.
#include <algorithm>
#include <cstring>

#include "chunk_internal.h"

namespace pmc {
namespace {

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t transit_bytes_of(const pmc_chunk_cfg& c) {
  return align256((size_t)c.seq * c.microbatch * c.hidden * (c.dtype == PMC_F32 ? 4 : 2));
}

// Largest number of inter-chunk buffers alive at once: a forward buffer lives from the F that
// writes it to the F of the next chunk, a backward buffer from a B to the B of the previous
// chunk.  One extra buffer receives outputs nobody reads.
int max_transit(const Schedule& s) {
  const int last = 2 * s.d - 1;
  int live = 0, peak = 0;
  for (const pmc_pass& p : s.passes) {
    if (p.op == PMC_F) {
      if (p.model_chunk < last) ++live;  // output buffer
      peak = std::max(peak, live);
      if (p.model_chunk > 0) --live;  // input buffer consumed
    } else if (p.op == PMC_B) {
      if (p.model_chunk > 0) ++live;
      peak = std::max(peak, live);
      if (p.model_chunk < last) --live;
    }
  }
  return peak + 1;
}

}  // namespace
}  // namespace pmc

using namespace pmc;

extern "C" {

size_t pmc_replay_workspace_bytes(const pmc_schedule* s, const pmc_chunk_cfg* cfg) {
  if (!s || !cfg) return 0;
  const size_t pass = pmc_pass_workspace_bytes(cfg);
  if (!pass) return 0;
  return align256(pass) + (size_t)max_transit(s->s) * transit_bytes_of(*cfg);
}

int schedule_replay(pmc_ctx* ctx, const pmc_schedule* sched, pmc_chunk* const* chunks, const void* const* x,
                    const void* const* dy_last, void* const* y_last, void* const* dx_first, uint32_t flags,
                    pmc_replay_report* report, pmc_device_peak* peaks, int32_t peaks_capacity) {
  if (!ctx || !sched || !chunks || !x || !dy_last || !report || !peaks)
    return fail(PMC_ERR_INVALID, "schedule_replay: NULL argument");
  const Schedule& s = sched->s;
  const int d = s.d, n = s.n, nchunks = 2 * d, last = nchunks - 1;
  if (peaks_capacity < d) return fail(PMC_ERR_INVALID, "schedule_replay: peaks capacity %d < d=%d", peaks_capacity, d);
  for (int c = 0; c < nchunks; ++c) {
    if (!chunks[c]) return fail(PMC_ERR_INVALID, "schedule_replay: chunk %d is NULL", c);
    if (chunk_ctx(chunks[c]) != ctx) return fail(PMC_ERR_INVALID, "schedule_replay: chunk %d belongs to another context", c);
    if (std::memcmp(&chunk_cfg(chunks[c]), &chunk_cfg(chunks[0]), sizeof(pmc_chunk_cfg)) != 0)
      return fail(PMC_ERR_INVALID, "schedule_replay: chunk %d differs in shape (uniform partition assumed)", c);
  }
  for (int j = 0; j < n; ++j)
    if (!x[j] || !dy_last[j]) return fail(PMC_ERR_INVALID, "schedule_replay: input %d is NULL", j);
  if (pmc_pool_live_slabs(ctx) != 0) return fail(PMC_ERR_STATE, "schedule_replay: pool has live slabs");

  const pmc_chunk_cfg& cfg = chunk_cfg(chunks[0]);
  const size_t pass_ws = align256(chunk_workspace_bytes(chunks[0]));
  const size_t tb = transit_bytes_of(cfg);
  const int ntransit = max_transit(s);
  size_t ws_bytes = 0;
  char* ws = ctx_workspace(ctx, &ws_bytes);
  if (!ws || ws_bytes < pass_ws + (size_t)ntransit * tb)
    return fail(PMC_ERR_NOMEM, "schedule_replay: workspace of %zu bytes, need %zu", ws_bytes, pass_ws + (size_t)ntransit * tb);

  // transit buffers: index 0 is the sink for outputs nobody reads
  std::vector<int> free_bufs;
  for (int i = ntransit - 1; i >= 1; --i) free_bufs.push_back(i);
  auto buf_ptr = [&](int i) { return (void*)(ws + pass_ws + (size_t)i * tb); };
  std::vector<int> fwd_buf((size_t)nchunks * n, -1), bwd_buf((size_t)nchunks * n, -1);
  int transit_live = 0, transit_peak = 0;
  auto take_buf = [&]() {
    if (free_bufs.empty()) return -1;  // cannot happen for a schedule max_transit() was computed from
    int b = free_bufs.back();
    free_bufs.pop_back();
    ++transit_live;
    transit_peak = std::max(transit_peak, transit_live);
    return b;
  };
  auto give_buf = [&](int b) {
    free_bufs.push_back(b);
    --transit_live;
  };

  hipStream_t st = ctx_stream(ctx);
  const bool time_passes = (flags & PMC_REPLAY_TIME_PASSES) != 0;
  hipEvent_t ev_begin = nullptr, ev_end = nullptr;
  std::vector<hipEvent_t> ev;
  bool running = false;  // passes are in flight: a failure must hand every held unit back
  auto cleanup = [&]() {
    if (running) {
      (void)hipStreamSynchronize(st);
      for (int c = 0; c < nchunks; ++c) chunk_release_all(chunks[c]);
      running = false;
    }
    if (ev_begin) (void)hipEventDestroy(ev_begin);
    if (ev_end) (void)hipEventDestroy(ev_end);
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  };
#define REPLAY_HIP(call)                                                                     \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess) {                                                                  \
      cleanup();                                                                             \
      return fail(PMC_ERR_HIP, "schedule_replay: %s: %s", #call, hipGetErrorString(e_));     \
    }                                                                                        \
  } while (0)
  REPLAY_HIP(hipEventCreate(&ev_begin));
  REPLAY_HIP(hipEventCreate(&ev_end));
  if (time_passes) {
    ev.resize(s.passes.size() + 1, nullptr);
    for (auto& e : ev) REPLAY_HIP(hipEventCreate(&e));
  }

  pmc_pool_reset_peak(ctx);
  int rc = PMC_OK;
  REPLAY_HIP(hipEventRecord(ev_begin, st));
  if (time_passes) REPLAY_HIP(hipEventRecord(ev[0], st));
  size_t done = 0;
  running = true;
  for (const pmc_pass& p : s.passes) {
    pmc_chunk* ch = chunks[p.model_chunk];
    const size_t slot = (size_t)p.model_chunk * n + p.mb;
    if (p.op == PMC_F) {
      if (s.grouped_bw && p.chunk == 0) {
        // 1F1B: the stage is the unit of allocation
        rc = chunk_reserve(ch, p.mb, p.device);
        if (rc == PMC_OK) rc = chunk_reserve(chunks[p.model_chunk + 1], p.mb, p.device);
        if (rc != PMC_OK) break;
      }
      const void* in = p.model_chunk == 0 ? x[p.mb] : buf_ptr(fwd_buf[slot - n]);
      void* out;
      if (p.model_chunk == last) {
        out = (y_last && y_last[p.mb]) ? y_last[p.mb] : buf_ptr(0);
      } else {
        fwd_buf[slot] = take_buf();
        if (fwd_buf[slot] < 0) {
          rc = fail(PMC_ERR_NOMEM, "schedule_replay: out of inter-chunk buffers");
          break;
        }
        out = buf_ptr(fwd_buf[slot]);
      }
      rc = chunk_forward(ch, p.mb, in, out, p.device);
      if (rc != PMC_OK) break;
      if (p.model_chunk > 0) {
        give_buf(fwd_buf[slot - n]);
        fwd_buf[slot - n] = -1;
      }
    } else if (p.op == PMC_B) {
      const void* in = p.model_chunk == last ? dy_last[p.mb] : buf_ptr(bwd_buf[slot + n]);
      void* out;
      if (p.model_chunk == 0) {
        out = (dx_first && dx_first[p.mb]) ? dx_first[p.mb] : buf_ptr(0);
      } else {
        bwd_buf[slot] = take_buf();
        if (bwd_buf[slot] < 0) {
          rc = fail(PMC_ERR_NOMEM, "schedule_replay: out of inter-chunk buffers");
          break;
        }
        out = buf_ptr(bwd_buf[slot]);
      }
      rc = chunk_backward_input(ch, p.mb, in, out);
      if (rc != PMC_OK) break;
      if (p.model_chunk < last) {
        give_buf(bwd_buf[slot + n]);
        bwd_buf[slot + n] = -1;
      }
    } else {
      if (s.grouped_bw) {
        // upper chunk's W keeps its unit until the lower chunk's W ends the fused backward
        rc = chunk_backward_weight_one(ch, p.mb, false);
        if (rc == PMC_OK && p.chunk == 0) {
          rc = chunk_release(ch, p.mb);
          if (rc == PMC_OK) rc = chunk_release(chunks[p.model_chunk + 1], p.mb);
        }
      } else {
        rc = chunk_backward_weight_one(ch, p.mb, true);
      }
      if (rc != PMC_OK) break;
    }
    ++done;
    if (time_passes) REPLAY_HIP(hipEventRecord(ev[done], st));
  }
  if (rc != PMC_OK) {
    // a pass failed: cleanup() waits for what was enqueued and returns every unit still held, so
    // that the pool is empty again and a later replay is not refused
    cleanup();
    return rc;
  }
  running = false;
  REPLAY_HIP(hipEventRecord(ev_end, st));
  REPLAY_HIP(hipStreamSynchronize(st));
  float ms = 0.f;
  REPLAY_HIP(hipEventElapsedTime(&ms, ev_begin, ev_end));
  std::memset(report, 0, sizeof(*report));
  report->ms_total = ms;
  report->passes = (int32_t)s.passes.size();
  report->devices = d;
  report->transit_peak_bytes = (int64_t)transit_peak * (int64_t)tb;
  if (time_passes) {
    for (size_t i = 0; i < s.passes.size(); ++i) {
      float t = 0.f;
      REPLAY_HIP(hipEventElapsedTime(&t, ev[i], ev[i + 1]));
      if (s.passes[i].op == PMC_F) report->ms_f += t;
      else if (s.passes[i].op == PMC_B) report->ms_b += t;
      else report->ms_w += t;
    }
  }
  ctx_device_peaks(ctx, d, (int64_t)chunk_unit_bytes(chunks[0]), peaks);
  cleanup();
  return PMC_OK;
#undef REPLAY_HIP
}

}  // extern "C"
