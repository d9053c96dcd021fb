// Host-only schedule generator: building blocks, repetition, pass orders, lifetime accounting
// and the as-early-as-possible timing of a squeezed schedule.  No HIP in this file.
//
// Construction (paper Section 2): the passes of one microbatch are laid out on a device x time
// grid; microbatch j's copy is shifted by j * T cells; a device's order is its passes sorted by
// cell, which squeezing preserves.  T = 6: every device runs 2 F, 2 B and 2 W per microbatch
// (Section 2.2: T equals the units of computation per stage of the block).
#include <algorithm>
#include <cstring>

#include "pmc_internal.h"

namespace pmc {
namespace {

constexpr int T = 6;
enum Row { F0 = 0, F1 = 1, B1 = 2, B0 = 3, W1 = 4, W0 = 5 };
const int kRowOp[6] = {PMC_F, PMC_F, PMC_B, PMC_B, PMC_W, PMC_W};
const int kRowChunk[6] = {0, 1, 1, 0, 1, 0};

// V-shape block (Section 3, 3.1): chunk 0 of device i is model chunk i, chunk 1 is 2d-1-i.
// Forward runs down the devices with step delta0, turns on the last device, runs back up with
// step delta1; the backward retraces it with the steps exchanged (Section 3.1's balance
// constraint delta_F^0 = delta_B^1, delta_F^1 = delta_B^0).
bool vshape_block(int d, int delta0, int delta1, int turn_f, int turn_fb, int turn_b,
                  std::vector<int32_t>& blk) {
  blk.assign(6 * d, 0);
  auto at = [&](int row, int i) -> int32_t& { return blk[row * d + i]; };
  for (int i = 0; i < d; ++i) at(F0, i) = i * delta0;
  at(F1, d - 1) = at(F0, d - 1) + turn_f;
  for (int i = d - 2; i >= 0; --i) at(F1, i) = at(F1, i + 1) + delta1;
  at(B1, 0) = at(F1, 0) + turn_fb;
  for (int i = 1; i < d; ++i) at(B1, i) = at(B1, i - 1) + delta0;
  at(B0, d - 1) = at(B1, d - 1) + turn_b;
  for (int i = d - 2; i >= 0; --i) at(B0, i) = at(B0, i + 1) + delta1;
  for (int i = 0; i < d; ++i) {
    bool used[T] = {false, false, false, false, false, false};
    for (int row : {F0, F1, B1, B0}) {
      int r = at(row, i) % T;
      if (used[r]) return false;  // would collide when repeated every T cells (Section 2.3)
      used[r] = true;
    }
    // W is placed greedily once F and B are settled (Section 3.1): in the order of the B passes,
    // each W takes the first cell after its B that is free modulo T.
    const int b_rows[2] = {B1, B0}, w_rows[2] = {W1, W0};
    for (int k = 0; k < 2; ++k) {
      int t = at(b_rows[k], i) + 1;
      while (used[t % T]) ++t;
      used[t % T] = true;
      at(w_rows[k], i) = t;
    }
  }
  return true;
}

// Two-part V-shape block of the adaptive scheduler (Appendix A, devices numbered 1..d there):
//   delta F_i^0 = delta B_i^1 = d0_lo for 1 <= i < K, d0_hi for K <= i < d;
//   delta F_i^1 = delta B_i^0 = d1_lo for 1 < i <= K, d1_hi for K < i <= d;
// K = d is the uniform block.  The same-device offsets pick the residue modulo T of each pass of
// the first device ("the permutation of the first device").
bool vshape_block_split(int d, int K, int d0_lo, int d1_lo, int d0_hi, int d1_hi, int turn_f, int turn_fb, int turn_b,
                        std::vector<int32_t>& blk) {
  blk.assign(6 * d, 0);
  auto at = [&](int row, int i) -> int32_t& { return blk[row * d + i]; };
  auto down = [&](int i) { return i + 1 < K ? d0_lo : d0_hi; };  // device i -> i + 1 (0-based i)
  auto up = [&](int i) { return i + 1 <= K ? d1_lo : d1_hi; };   // device i -> i - 1
  for (int i = 0; i + 1 < d; ++i) at(F0, i + 1) = at(F0, i) + down(i);
  at(F1, d - 1) = at(F0, d - 1) + turn_f;
  for (int i = d - 1; i > 0; --i) at(F1, i - 1) = at(F1, i) + up(i);
  at(B1, 0) = at(F1, 0) + turn_fb;
  for (int i = 0; i + 1 < d; ++i) at(B1, i + 1) = at(B1, i) + down(i);
  at(B0, d - 1) = at(B1, d - 1) + turn_b;
  for (int i = d - 1; i > 0; --i) at(B0, i - 1) = at(B0, i) + up(i);
  for (int i = 0; i < d; ++i) {
    bool used[T] = {false, false, false, false, false, false};
    for (int row : {F0, F1, B1, B0}) {
      int r = at(row, i) % T;
      if (used[r]) return false;
      used[r] = true;
    }
    const int b_rows[2] = {B1, B0}, w_rows[2] = {W1, W0};
    for (int k = 0; k < 2; ++k) {
      int t = at(b_rows[k], i) + 1;
      while (used[t % T]) ++t;
      used[t % T] = true;
      at(w_rows[k], i) = t;
    }
  }
  return true;
}

// Largest number of live units any device reaches when the block is repeated for n microbatches:
// the live count can only peak when an F starts, and a unit of chunk c, microbatch j is live in
// cells F_c + jT .. W_c + jT.
int64_t block_peak_units(const std::vector<int32_t>& blk, int d, int n) {
  const int f_rows[2] = {F0, F1}, w_rows[2] = {W0, W1};
  int64_t peak = 0;
  for (int i = 0; i < d; ++i)
    for (int c = 0; c < 2; ++c)
      for (int j = 0; j < n; ++j) {
        const int64_t t = blk[f_rows[c] * d + i] + (int64_t)j * T;
        int64_t live = 0;
        for (int c2 = 0; c2 < 2; ++c2) {
          const int64_t f = blk[f_rows[c2] * d + i], w = blk[w_rows[c2] * d + i];
          // microbatches j2 with f + j2 T <= t <= w + j2 T
          int64_t hi = (t - f) >= 0 ? (t - f) / T : -1;
          int64_t lo = (t - w) > 0 ? (t - w + T - 1) / T : 0;
          hi = std::min<int64_t>(hi, n - 1);
          if (hi >= lo) live += hi - lo + 1;
        }
        peak = std::max(peak, live);
      }
  return peak;
}

// 1F1B at chunk granularity: a stage (two consecutive chunks) runs F of both chunks in two cells
// and its fused backward in four (B, W of the upper chunk, then of the lower one).  Adjacent
// stages' forwards are 2 cells apart, their backwards 4 (Table 1's delta0, delta1 for 1F1B).
void one_f_one_b_block(int d, std::vector<int32_t>& blk) {
  blk.assign(6 * d, 0);
  for (int i = 0; i < d; ++i) {
    int tf = 2 * i, tbw = 2 * d + 4 * (d - 1 - i);
    blk[F0 * d + i] = tf;
    blk[F1 * d + i] = tf + 1;
    blk[B1 * d + i] = tbw;
    blk[W1 * d + i] = tbw + 1;
    blk[B0 * d + i] = tbw + 2;
    blk[W0 * d + i] = tbw + 3;
  }
}

// 1F1B-V (Appendix H): V-shape placement of 1F1B's block without the B/W split.  A chunk's backward
// is one pass of two cells (B, W); a pass that depends on it waits for its end.  Earliest fit: F of
// the first half down the devices, F of the second half up, the fused backward of the second half
// down, of the first half up, each at the first cell at or after its dependency's end where its own
// cells are free modulo T on its device AND the device's passes still to come can be packed into
// what stays free (the six residues of a device end up exactly filled: 1 + 1 + 2 + 2).
// `f_turn` delays the forward's turn on the last device by that many cells.
void one_f_one_b_v_block_at(int d, int f_turn, std::vector<int32_t>& blk) {
  blk.assign(6 * d, 0);
  std::vector<unsigned> free_mask(d, (1u << T) - 1);
  auto cells_of = [](int t, int len) {
    unsigned m = 0;
    for (int k = 0; k < len; ++k) m |= 1u << ((t + k) % T);
    return m;
  };
  // can runs of these lengths (at most two of them, in any position) be cut out of the mask?
  auto packs = [&](unsigned mask, const int* len, int count) {
    if (count == 0) return true;
    for (int r = 0; r < T; ++r) {
      const unsigned a = cells_of(r, len[0]);
      if ((mask & a) != a) continue;
      if (count == 1) return true;
      const unsigned rest = mask & ~a;
      for (int q = 0; q < T; ++q) {
        const unsigned b = cells_of(q, len[1]);
        if ((rest & b) != b) continue;
        if (count == 2) return true;
        const unsigned rest2 = rest & ~b;
        for (int u = 0; u < T; ++u) {
          const unsigned c = cells_of(u, len[2]);
          if ((rest2 & c) == c) return true;
        }
      }
    }
    return false;
  };
  auto place = [&](int i, int ready, int len, const int* later, int nlater) {
    for (int t = ready;; ++t) {
      const unsigned m = cells_of(t, len);
      if ((free_mask[i] & m) == m && packs(free_mask[i] & ~m, later, nlater)) {
        free_mask[i] &= ~m;
        return t;
      }
    }
  };
  const int after_f0[3] = {1, 2, 2}, after_f1[2] = {2, 2}, after_b1[1] = {2};
  auto at = [&](int row, int i) -> int32_t& { return blk[row * d + i]; };
  for (int i = 0; i < d; ++i) at(F0, i) = place(i, i == 0 ? 0 : at(F0, i - 1) + 1, 1, after_f0, 3);
  for (int i = d - 1; i >= 0; --i) at(F1, i) = place(i, (i == d - 1 ? at(F0, d - 1) + f_turn : at(F1, i + 1)) + 1, 1, after_f1, 2);
  for (int i = 0; i < d; ++i) at(B1, i) = place(i, i == 0 ? at(F1, 0) + 1 : at(B1, i - 1) + 2, 2, after_b1, 1);
  for (int i = d - 1; i >= 0; --i) at(B0, i) = place(i, (i == d - 1 ? at(B1, d - 1) : at(B0, i + 1)) + 2, 2, nullptr, 0);
  for (int i = 0; i < d; ++i) {
    at(W1, i) = at(B1, i) + 1;
    at(W0, i) = at(B0, i) + 1;
  }
}

int model_chunk(const Schedule& s, int device, int chunk) {
  if (s.grouped_bw) return 2 * device + chunk;
  return chunk == 0 ? device : 2 * s.d - 1 - device;
}

int finish(Schedule& s) {
  const int d = s.d, n = s.n;
  s.per_device.assign(d, {});
  for (int i = 0; i < d; ++i) {
    auto& v = s.per_device[i];
    v.reserve(6 * n);
    for (int row = 0; row < 6; ++row)
      for (int j = 0; j < n; ++j) {
        pmc_pass p;
        p.time = s.block[row * d + i] + j * T;
        p.device = i;
        p.op = kRowOp[row];
        p.chunk = kRowChunk[row];
        p.mb = j;
        p.model_chunk = model_chunk(s, i, p.chunk);
        v.push_back(p);
      }
    std::sort(v.begin(), v.end(), [](const pmc_pass& a, const pmc_pass& b) { return a.time < b.time; });
    for (size_t k = 1; k < v.size(); ++k)
      if (v[k].time == v[k - 1].time)
        return fail(PMC_ERR_ILLEGAL_BLOCK, "two passes share cell %d on device %d", v[k].time, i);
  }
  s.passes.clear();
  for (auto& v : s.per_device) s.passes.insert(s.passes.end(), v.begin(), v.end());
  std::sort(s.passes.begin(), s.passes.end(), [](const pmc_pass& a, const pmc_pass& b) {
    return a.time != b.time ? a.time < b.time : a.device < b.device;
  });
  return PMC_OK;
}

}  // namespace

int makespan(const Schedule& s, double tf, double tb, double tw, double* out);
void account(const Schedule& s, int64_t unit_bytes, int64_t stats_bytes, pmc_device_peak* out);

// The free parameter of the 1F1B-V block, chosen as the paper chooses V-ZB's same-device offsets
// (brute force, Section 3.1): least peak of live units, then least unit-time makespan, with 3d
// microbatches; the first such delay in 0 .. T-1.
int one_f_one_b_v_block(int d, std::vector<int32_t>& blk) {
  bool have = false;
  int64_t best_peak = 0;
  double best_span = 0.0;
  Schedule trial;
  trial.kind = PMC_1F1BV;
  trial.d = d;
  trial.n = 3 * d;
  trial.fused = true;
  std::vector<pmc_device_peak> peaks(d);
  for (int a = 0; a < T; ++a) {
    one_f_one_b_v_block_at(d, a, trial.block);
    if (int rc = finish(trial)) return rc;
    account(trial, 1, 0, peaks.data());
    int64_t peak = 0;
    for (const auto& p : peaks) peak = std::max(peak, p.peak_live_units);
    double span = 0.0;
    if (int rc = makespan(trial, 1.0, 1.0, 1.0, &span)) return rc;
    if (!have || peak < best_peak || (peak == best_peak && span < best_span)) {
      have = true;
      best_peak = peak;
      best_span = span;
      blk = trial.block;
    }
  }
  return PMC_OK;
}

int build_schedule(int kind, int d, int n, Schedule& s) {
  if (d < 1 || n < 1) return fail(PMC_ERR_INVALID, "need d >= 1 and n >= 1 (got d=%d n=%d)", d, n);
  if ((int64_t)d * n > (1 << 24)) return fail(PMC_ERR_INVALID, "d*n too large");
  s.kind = kind;
  s.d = d;
  s.n = n;
  s.grouped_bw = false;
  s.fused = false;
  bool ok = true;
  switch (kind) {
    case PMC_1F1B:
      s.grouped_bw = true;
      s.fused = true;
      one_f_one_b_block(d, s.block);
      break;
    case PMC_1F1BV:
      s.fused = true;
      if (int rc = one_f_one_b_v_block(d, s.block)) return rc;
      break;
    case PMC_VMIN:  // Table 1 (1,1); Appendix F: F->B turn is 3 when d is a multiple of 3
      ok = vshape_block(d, 1, 1, 1, d % 3 == 0 ? 3 : 1, 1, s.block);
      break;
    case PMC_VHALF:  // Table 1 (2,1); Appendix F: F turn 2, F->B turn 4 for even d
      ok = vshape_block(d, 2, 1, 2, d % 2 == 0 ? 4 : 1, 1, s.block);
      break;
    case PMC_VZB:  // Table 1 (4,2); same-device offsets not printed in the paper
      ok = vshape_block(d, 4, 2, 1, 1, 1, s.block);
      break;
    default:
      return fail(PMC_ERR_INVALID, "unknown schedule kind %d", kind);
  }
  if (!ok) return fail(PMC_ERR_ILLEGAL_BLOCK, "building block of kind %d collides for d=%d", kind, d);
  return finish(s);
}

int build_vshape(int d, int n, int delta0, int delta1, int turn_f, int turn_fb, int turn_b, Schedule& s) {
  if (d < 1 || n < 1) return fail(PMC_ERR_INVALID, "need d >= 1 and n >= 1");
  if (delta0 < 1 || delta1 < 1 || turn_f < 1 || turn_fb < 1 || turn_b < 1)
    return fail(PMC_ERR_INVALID, "offsets must be positive");
  s.kind = -1;
  s.d = d;
  s.n = n;
  s.grouped_bw = false;
  s.fused = false;
  if (!vshape_block(d, delta0, delta1, turn_f, turn_fb, turn_b, s.block))
    return fail(PMC_ERR_ILLEGAL_BLOCK, "V-shape block (%d,%d | %d,%d,%d) collides for d=%d", delta0, delta1,
                turn_f, turn_fb, turn_b, d);
  return finish(s);
}

// Section 2.2: a unit is allocated when its F starts and retained until B and W have both used
// it.  With 1F1B the stage is the unit: two chunk units from the start of the stage's F to the
// end of its fused backward.
void account(const Schedule& s, int64_t unit_bytes, int64_t stats_bytes, pmc_device_peak* out) {
  for (int i = 0; i < s.d; ++i) {
    int64_t units = 0, peak_units = 0, bytes = 0, peak_bytes = 0;
    for (const pmc_pass& p : s.per_device[i]) {
      if (p.op == PMC_F) {
        if (!s.grouped_bw) {
          units += 1;
          bytes += unit_bytes;
        } else if (p.chunk == 0) {
          units += 2;
          bytes += 2 * unit_bytes;
        }
        peak_units = std::max(peak_units, units);
        peak_bytes = std::max(peak_bytes, bytes);
      } else if (p.op == PMC_B) {
        bytes -= stats_bytes;
      } else {
        if (!s.grouped_bw) {
          units -= 1;
          bytes -= unit_bytes - stats_bytes;
        } else if (p.chunk == 0) {
          units -= 2;
          bytes -= 2 * (unit_bytes - stats_bytes);
        }
      }
    }
    out[i].peak_live_units = peak_units;
    out[i].peak_live_bytes = peak_units * unit_bytes;
    out[i].peak_tensor_bytes = peak_bytes;
  }
}

// Every device starts each pass of its order as soon as the device is free and the passes it
// depends on have ended.  F needs F of the previous model chunk, B needs B of the next one (the
// last chunk's B needs its own F), W needs its own B.  In 1F1B the backward of a stage is one
// pass, so the stage before it waits for the end of that whole pass; likewise in 1F1B-V, chunk by chunk.
int makespan(const Schedule& s, double tf, double tb, double tw, double* out) {
  const int d = s.d, n = s.n, last = 2 * d - 1;
  const double dur[3] = {tf, tb, tw};
  std::vector<double> end((size_t)3 * 2 * d * n, -1.0);
  auto idx = [&](int op, int mc, int mb) { return ((size_t)op * 2 * d + mc) * n + mb; };
  std::vector<size_t> next(d, 0);
  std::vector<double> free_at(d, 0.0);
  size_t remaining = s.passes.size();
  while (remaining) {
    bool progressed = false;
    for (int i = 0; i < d; ++i) {
      while (next[i] < s.per_device[i].size()) {
        const pmc_pass& p = s.per_device[i][next[i]];
        int dep_op = -1, dep_mc = 0;
        if (p.op == PMC_F) {
          if (p.model_chunk > 0) dep_op = PMC_F, dep_mc = p.model_chunk - 1;
        } else if (p.op == PMC_B) {
          if (p.model_chunk == last) dep_op = PMC_F, dep_mc = last;
          else if (s.fused && (!s.grouped_bw || p.chunk == 1)) dep_op = PMC_W, dep_mc = p.model_chunk + 1;
          else dep_op = PMC_B, dep_mc = p.model_chunk + 1;
        } else {
          dep_op = PMC_B, dep_mc = p.model_chunk;
        }
        double start = free_at[i];
        if (dep_op >= 0) {
          double e = end[idx(dep_op, dep_mc, p.mb)];
          if (e < 0) break;
          start = std::max(start, e);
        }
        free_at[i] = end[idx(p.op, p.model_chunk, p.mb)] = start + dur[p.op];
        ++next[i];
        --remaining;
        progressed = true;
      }
    }
    if (!progressed) return fail(PMC_ERR_ILLEGAL_BLOCK, "orders contradict the dependencies");
  }
  *out = *std::max_element(free_at.begin(), free_at.end());
  return PMC_OK;
}

namespace {

// Integer-cell view of a schedule at unit pass times, used by the reordering heuristics.
struct Grid {
  int d, n, last;
  bool fused, grouped;
  std::vector<int32_t> end;  // [3][2d][n]: end cell of (op, model chunk, microbatch), -1 = not placed
  size_t idx(int op, int mc, int mb) const { return ((size_t)op * 2 * d + mc) * n + mb; }
  // the one pass p waits for, or op = -1
  void dependency(const pmc_pass& p, int& op, int& mc) const {
    op = -1;
    mc = 0;
    if (p.op == PMC_F) {
      if (p.model_chunk > 0) op = PMC_F, mc = p.model_chunk - 1;
    } else if (p.op == PMC_B) {
      if (p.model_chunk == last) op = PMC_F, mc = last;
      else if (fused && (!grouped || p.chunk == 1)) op = PMC_W, mc = p.model_chunk + 1;
      else op = PMC_B, mc = p.model_chunk + 1;
    } else {
      op = PMC_B, mc = p.model_chunk;
    }
  }
};

// Squeezes the given per-device orders at unit times: writes every pass's start cell into
// pass.time and its end into g.end.  False if the orders contradict the dependencies.
bool squeeze_unit(Grid& g, std::vector<std::vector<pmc_pass>>& orders) {
  std::fill(g.end.begin(), g.end.end(), -1);
  std::vector<size_t> next(g.d, 0);
  std::vector<int32_t> free_at(g.d, 0);
  size_t remaining = 0;
  for (auto& o : orders) remaining += o.size();
  while (remaining) {
    bool progressed = false;
    for (int i = 0; i < g.d; ++i) {
      while (next[i] < orders[i].size()) {
        pmc_pass& p = orders[i][next[i]];
        int op, mc;
        g.dependency(p, op, mc);
        int32_t start = free_at[i];
        if (op >= 0) {
          const int32_t e = g.end[g.idx(op, mc, p.mb)];
          if (e < 0) break;
          start = std::max(start, e);
        }
        p.time = start;
        free_at[i] = g.end[g.idx(p.op, p.model_chunk, p.mb)] = start + 1;
        ++next[i];
        --remaining;
        progressed = true;
      }
    }
    if (!progressed) return false;
  }
  return true;
}

int64_t peak_units_of(const std::vector<pmc_pass>& order) {
  int64_t live = 0, peak = 0;
  for (const pmc_pass& p : order) {
    if (p.op == PMC_F) peak = std::max(peak, ++live);
    else if (p.op == PMC_W) --live;
  }
  return peak;
}

void sort_by_cell(std::vector<pmc_pass>& v) {
  std::sort(v.begin(), v.end(), [](const pmc_pass& a, const pmc_pass& b) { return a.time < b.time; });
}

}  // namespace

// Section 2 "Reordering" with the two greedy heuristics of Appendix C, on the squeezed grid at
// unit pass times.  Warm-up: vacant cells before a device's first B are filled, left to right, with
// the first later pass of that device whose dependency has ended, all other passes staying put; a
// move that would raise the device's peak of live units is refused (the reordering is stated to
// leave the peak unchanged).  Cool-down: the W passes after a device's last F are taken out, the
// rest is squeezed, and the vacant cells after the last F are filled left to right with the first
// removed W whose B has ended; the remainder goes to the end.  The result's `time` fields are the
// cells of the final squeezed grid.  A fused-backward (1F1B, 1F1B-V) schedule is only squeezed.
int reorder(const Schedule& in, Schedule& out) {
  out = in;
  const int d = in.d, n = in.n;
  Grid g{d, n, 2 * d - 1, in.fused, in.grouped_bw, std::vector<int32_t>((size_t)3 * 2 * d * n, -1)};
  auto& orders = out.per_device;
  if (!squeeze_unit(g, orders)) return fail(PMC_ERR_ILLEGAL_BLOCK, "orders contradict the dependencies");
  if (!in.fused) {
    std::vector<int64_t> base_peak(d);
    std::vector<int32_t> first_b(d, 0);
    int32_t horizon = 0;
    for (int i = 0; i < d; ++i) {
      base_peak[i] = peak_units_of(orders[i]);
      for (const pmc_pass& p : orders[i])
        if (p.op == PMC_B) {
          first_b[i] = p.time;
          break;
        }
      horizon = std::max(horizon, first_b[i]);
    }
    // warm-up: orders[i] stays sorted by cell throughout
    for (int32_t t = 0; t < horizon; ++t)
      for (int i = 0; i < d; ++i) {
        if (t >= first_b[i]) continue;
        auto& o = orders[i];
        auto at = std::lower_bound(o.begin(), o.end(), t, [](const pmc_pass& p, int32_t c) { return p.time < c; });
        if (at != o.end() && at->time == t) continue;  // occupied
        const size_t pos = at - o.begin();               // the moved pass is inserted here
        for (size_t k = pos; k < o.size(); ++k) {
          pmc_pass p = o[k];
          int op, mc;
          g.dependency(p, op, mc);
          if (op >= 0 && g.end[g.idx(op, mc, p.mb)] > t) continue;
          std::vector<pmc_pass> trial(o);
          trial.erase(trial.begin() + k);
          p.time = t;
          trial.insert(trial.begin() + pos, p);
          if (peak_units_of(trial) > base_peak[i]) continue;
          o.swap(trial);
          g.end[g.idx(p.op, p.model_chunk, p.mb)] = t + 1;
          break;
        }
      }
    if (!squeeze_unit(g, orders)) return fail(PMC_ERR_ILLEGAL_BLOCK, "warm-up reordering broke a dependency");
    // cool-down
    std::vector<std::vector<pmc_pass>> removed(d);
    for (int i = 0; i < d; ++i) {
      auto& o = orders[i];
      size_t last_f = 0;
      for (size_t k = 0; k < o.size(); ++k)
        if (o[k].op == PMC_F) last_f = k;
      std::vector<pmc_pass> kept;
      for (size_t k = 0; k < o.size(); ++k) {
        if (o[k].op == PMC_W && k > last_f) removed[i].push_back(o[k]);
        else kept.push_back(o[k]);
      }
      o.swap(kept);
    }
    if (!squeeze_unit(g, orders)) return fail(PMC_ERR_ILLEGAL_BLOCK, "cool-down reordering broke a dependency");
    for (int i = 0; i < d; ++i) {
      auto& o = orders[i];
      int32_t t = 0;
      for (const pmc_pass& p : o)
        if (p.op == PMC_F) t = p.time + 1;
      std::vector<pmc_pass>& pending = removed[i];
      size_t scan = 0;  // first kept pass at or after cell t
      while (scan < o.size() && o[scan].time < t) ++scan;
      std::vector<pmc_pass> placed;
      while (!pending.empty()) {
        if (scan < o.size() && o[scan].time == t) {
          ++scan;
        } else {
          for (size_t k = 0; k < pending.size(); ++k)
            if (g.end[g.idx(PMC_B, pending[k].model_chunk, pending[k].mb)] <= t) {
              pmc_pass w = pending[k];
              w.time = t;
              placed.push_back(w);
              pending.erase(pending.begin() + k);
              break;
            }
        }
        ++t;
      }
      o.insert(o.end(), placed.begin(), placed.end());
      sort_by_cell(o);
    }
    if (!squeeze_unit(g, orders)) return fail(PMC_ERR_ILLEGAL_BLOCK, "reordering broke a dependency");
  }
  out.passes.clear();
  for (auto& v : orders) out.passes.insert(out.passes.end(), v.begin(), v.end());
  std::sort(out.passes.begin(), out.passes.end(), [](const pmc_pass& a, const pmc_pass& b) {
    return a.time != b.time ? a.time < b.time : a.device < b.device;
  });
  return PMC_OK;
}

// Adaptive scheduler (Appendix A): every two-part block within the offset range, in a fixed
// order; blocks that collide or whose peak exceeds the limit are dropped; the rest are repeated,
// squeezed, optionally reordered and timed with the given pass times; the first block with the
// least finish time wins.
int search(int d, int n, int64_t limit_units, double tf, double tb, double tw, int max_delta, bool do_reorder,
           pmc_search_result* res, Schedule& best) {
  if (d < 1 || n < 1) return fail(PMC_ERR_INVALID, "need d >= 1 and n >= 1 (got d=%d n=%d)", d, n);
  if ((int64_t)d * n > (1 << 20)) return fail(PMC_ERR_INVALID, "d*n too large for a search");
  if (max_delta < 1 || max_delta > 4 * T) return fail(PMC_ERR_INVALID, "max_delta %d out of range", max_delta);
  if (tf < 0 || tb < 0 || tw < 0) return fail(PMC_ERR_INVALID, "negative duration");
  bool found = false;
  double best_span = 0.0;
  int64_t candidates = 0, feasible = 0;
  Schedule cand, reordered;
  for (int K = d > 1 ? 2 : 1; K <= d; ++K)
    for (int d0_lo = 1; d0_lo <= max_delta; ++d0_lo)
      for (int d1_lo = 1; d1_lo <= max_delta; ++d1_lo)
        for (int d0_hi = (K < d ? 1 : d0_lo); d0_hi <= (K < d ? max_delta : d0_lo); ++d0_hi)
          for (int d1_hi = (K < d ? 1 : d1_lo); d1_hi <= (K < d ? max_delta : d1_lo); ++d1_hi)
            for (int a = 1; a <= T; ++a)
              for (int b = 1; b <= T; ++b)
                for (int c = 1; c <= T; ++c) {
                  ++candidates;
                  if (!vshape_block_split(d, K, d0_lo, d1_lo, d0_hi, d1_hi, a, b, c, cand.block)) continue;
                  const int64_t peak = block_peak_units(cand.block, d, n);
                  if (peak > limit_units) continue;
                  ++feasible;
                  cand.kind = -1;
                  cand.d = d;
                  cand.n = n;
                  cand.grouped_bw = false;
                  cand.fused = false;
                  if (int rc = finish(cand)) return rc;
                  const Schedule* timed = &cand;
                  if (do_reorder) {
                    if (int rc = reorder(cand, reordered)) return rc;
                    timed = &reordered;
                  }
                  double span = 0.0;
                  if (int rc = makespan(*timed, tf, tb, tw, &span)) return rc;
                  if (!found || span < best_span) {
                    found = true;
                    best_span = span;
                    best = *timed;
                    if (res) {
                      res->split = K;
                      res->delta0_lo = d0_lo;
                      res->delta1_lo = d1_lo;
                      res->delta0_hi = d0_hi;
                      res->delta1_hi = d1_hi;
                      res->turn_f = a;
                      res->turn_fb = b;
                      res->turn_b = c;
                      res->peak_units = peak;
                      res->makespan = span;
                    }
                  }
                }
  if (res) {
    res->candidates = candidates;
    res->feasible = feasible;
  }
  if (!found) return fail(PMC_ERR_ILLEGAL_BLOCK, "no V-shape block with offsets up to %d fits %lld live units on d=%d", max_delta,
                          (long long)limit_units, d);
  return PMC_OK;
}

}  // namespace pmc

using pmc::fail;

extern "C" {

int pmc_schedule_build(int32_t kind, int32_t d, int32_t n, pmc_schedule** out) {
  if (!out) return fail(PMC_ERR_INVALID, "out is NULL");
  auto* s = new (std::nothrow) pmc_schedule;
  if (!s) return fail(PMC_ERR_NOMEM, "host allocation failed");
  int rc = pmc::build_schedule(kind, d, n, s->s);
  if (rc != PMC_OK) {
    delete s;
    return rc;
  }
  *out = s;
  return PMC_OK;
}

int pmc_schedule_build_vshape(int32_t d, int32_t n, int32_t delta0, int32_t delta1, int32_t turn_f,
                              int32_t turn_fb, int32_t turn_b, pmc_schedule** out) {
  if (!out) return fail(PMC_ERR_INVALID, "out is NULL");
  auto* s = new (std::nothrow) pmc_schedule;
  if (!s) return fail(PMC_ERR_NOMEM, "host allocation failed");
  int rc = pmc::build_vshape(d, n, delta0, delta1, turn_f, turn_fb, turn_b, s->s);
  if (rc != PMC_OK) {
    delete s;
    return rc;
  }
  *out = s;
  return PMC_OK;
}

int pmc_schedule_reorder(const pmc_schedule* s, pmc_schedule** out) {
  if (!s || !out) return fail(PMC_ERR_INVALID, "NULL argument");
  auto* r = new (std::nothrow) pmc_schedule;
  if (!r) return fail(PMC_ERR_NOMEM, "host allocation failed");
  int rc = pmc::reorder(s->s, r->s);
  if (rc != PMC_OK) {
    delete r;
    return rc;
  }
  *out = r;
  return PMC_OK;
}

int pmc_schedule_search(int32_t d, int32_t n, int64_t limit_units, double t_f, double t_b, double t_w, int32_t max_delta,
                        int32_t reorder, pmc_search_result* result, pmc_schedule** out) {
  if (!out) return fail(PMC_ERR_INVALID, "out is NULL");
  auto* s = new (std::nothrow) pmc_schedule;
  if (!s) return fail(PMC_ERR_NOMEM, "host allocation failed");
  int rc = pmc::search(d, n, limit_units, t_f, t_b, t_w, max_delta, reorder != 0, result, s->s);
  if (rc != PMC_OK) {
    delete s;
    return rc;
  }
  *out = s;
  return PMC_OK;
}

void pmc_schedule_destroy(pmc_schedule* s) { delete s; }
int32_t pmc_schedule_devices(const pmc_schedule* s) { return s ? s->s.d : 0; }
int32_t pmc_schedule_microbatches(const pmc_schedule* s) { return s ? s->s.n : 0; }
int32_t pmc_schedule_num_passes(const pmc_schedule* s) { return s ? (int32_t)s->s.passes.size() : 0; }

int pmc_schedule_block(const pmc_schedule* s, int32_t* out, int32_t capacity) {
  if (!s || !out) return fail(PMC_ERR_INVALID, "NULL argument");
  if (capacity < (int32_t)s->s.block.size()) return fail(PMC_ERR_INVALID, "capacity %d < %zu", capacity, s->s.block.size());
  std::memcpy(out, s->s.block.data(), s->s.block.size() * sizeof(int32_t));
  return PMC_OK;
}

int pmc_schedule_device_order(const pmc_schedule* s, int32_t device, pmc_pass* out, int32_t capacity) {
  if (!s || !out) return fail(PMC_ERR_INVALID, "NULL argument");
  if (device < 0 || device >= s->s.d) return fail(PMC_ERR_INVALID, "device %d out of range", device);
  const auto& v = s->s.per_device[device];
  if (capacity < (int32_t)v.size()) return fail(PMC_ERR_INVALID, "capacity %d < %zu", capacity, v.size());
  std::memcpy(out, v.data(), v.size() * sizeof(pmc_pass));
  return PMC_OK;
}

int pmc_schedule_global_order(const pmc_schedule* s, pmc_pass* out, int32_t capacity) {
  if (!s || !out) return fail(PMC_ERR_INVALID, "NULL argument");
  const auto& v = s->s.passes;
  if (capacity < (int32_t)v.size()) return fail(PMC_ERR_INVALID, "capacity %d < %zu", capacity, v.size());
  std::memcpy(out, v.data(), v.size() * sizeof(pmc_pass));
  return PMC_OK;
}

int pmc_schedule_account(const pmc_schedule* s, int64_t unit_bytes, int64_t stats_bytes, pmc_device_peak* out,
                         int32_t capacity) {
  if (!s || !out) return fail(PMC_ERR_INVALID, "NULL argument");
  if (capacity < s->s.d) return fail(PMC_ERR_INVALID, "capacity %d < d=%d", capacity, s->s.d);
  if (unit_bytes < 0 || stats_bytes < 0 || stats_bytes > unit_bytes) return fail(PMC_ERR_INVALID, "bad byte sizes");
  pmc::account(s->s, unit_bytes, stats_bytes, out);
  return PMC_OK;
}

int pmc_schedule_makespan(const pmc_schedule* s, double t_f, double t_b, double t_w, double* out) {
  if (!s || !out) return fail(PMC_ERR_INVALID, "NULL argument");
  if (t_f < 0 || t_b < 0 || t_w < 0) return fail(PMC_ERR_INVALID, "negative duration");
  return pmc::makespan(s->s, t_f, t_b, t_w, out);
}

}  // extern "C"
