// Host side of the library: context, activation pool, workspace, chunks and the three passes
// F / B / W of a chunk (paper Section 2.1), plus the single-operation entry points.
//
// What one (chunk, microbatch) keeps between its F and its W lives in ONE slab of the pool
// (Section 2.2: allocated when F starts, retained until B and W have both consumed it).  Per
// layer the slab holds, in the storage type,
//     X  A  QKV  O  XMID  C  U  G        (h, h, 3h, h, h, h, ffn, ffn columns)
// and after all layers the fp32 statistics (LayerNorm mean/rstd twice, attention log-sum-exp).
// B overwrites what only it needs with what W needs, one for one:
//     U <- dU (GeLU' epilogue, in place),  XMID <- dX_mid,  QKV <- dQKV,
//     X[l+1] <- dX of layer l+1 (= dX_out of layer l),  X[0] <- dY of the chunk,
// so the slab never grows.  Tensors that exist only inside B (dC, dO, dA, the dQ staging buffer,
// partial sums) live in the workspace.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <set>

#include "kernels.h"

namespace pmc {

namespace {
size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
}  // namespace

struct Pool {
  char* base = nullptr;
  size_t slab_bytes = 0;
  int64_t slabs = 0;
  std::set<int64_t> free_list;  // lowest index first: placement is deterministic
  int64_t live = 0, peak = 0;
  struct Dev {
    int64_t units = 0, peak_units = 0, tensor_bytes = 0, peak_tensor_bytes = 0;
  };
  std::map<int, Dev> dev;

  void* take(int device, int64_t unit_bytes) {
    if (free_list.empty()) return nullptr;
    int64_t i = *free_list.begin();
    free_list.erase(free_list.begin());
    ++live;
    peak = std::max(peak, live);
    Dev& d = dev[device];
    d.units += 1;
    d.tensor_bytes += unit_bytes;
    d.peak_units = std::max(d.peak_units, d.units);
    d.peak_tensor_bytes = std::max(d.peak_tensor_bytes, d.tensor_bytes);
    return base + (size_t)i * slab_bytes;
  }
  void shrink(int device, int64_t bytes) { dev[device].tensor_bytes -= bytes; }
  void give(void* p, int device, int64_t remaining_bytes) {
    free_list.insert(((char*)p - base) / (int64_t)slab_bytes);
    --live;
    Dev& d = dev[device];
    d.units -= 1;
    d.tensor_bytes -= remaining_bytes;
  }
  void reset_peaks() {
    peak = live;
    for (auto& kv : dev) {
      kv.second.peak_units = kv.second.units;
      kv.second.peak_tensor_bytes = kv.second.tensor_bytes;
    }
  }
};

}  // namespace pmc

namespace pmc {
struct TraceSlot {
  pmc_trace_rec rec;
  hipEvent_t e0, e1;
};
}  // namespace pmc

struct pmc_ctx {
  hipStream_t stream = nullptr;
  bool tracing = false;
  size_t trace_capacity = 0;
  std::vector<pmc::TraceSlot> trace;
  pmc::Pool pool;
  char* ws = nullptr;
  size_t ws_bytes = 0;
  int chunks_alive = 0;
  // second stream for the W pass (created on first use, default priority)
  static constexpr int kSide = 1;
  hipStream_t side[kSide] = {};
  hipEvent_t fork = nullptr, join[kSide] = {};
  ~pmc_ctx() {
    if (fork) (void)hipEventDestroy(fork);
    for (int i = 0; i < kSide; ++i) {
      if (join[i]) (void)hipEventDestroy(join[i]);
      if (side[i]) (void)hipStreamDestroy(side[i]);
    }
  }
};

namespace pmc {

enum MbState { kReserved = 0, kForwardDone = 1, kBackwardDone = 2 };

struct Micro {
  char* slab = nullptr;
  int state = kReserved;
  int device = 0;
};

struct LayerOffsets {  // byte offsets inside the slab
  size_t x, a, qkv, o, xmid, c, u, g;
  size_t mean1, rstd1, mean2, rstd2, lse;
};

struct WorkspaceLayout {
  size_t t_h, attn, partial, partial_stride, gemm, gemm_bytes, total;
};

}  // namespace pmc

struct pmc_chunk {
  pmc_ctx* ctx = nullptr;
  pmc_chunk_cfg cfg{};
  int tokens = 0, head_dim = 0;
  size_t esz = 0;
  size_t unit_bytes = 0, stats_bytes = 0;
  std::vector<pmc::LayerOffsets> off;
  pmc::WorkspaceLayout wsl{};
  std::vector<const void*> params;
  std::vector<float*> grads;
  bool bound = false;
  std::map<int32_t, pmc::Micro> live;
};

namespace pmc {
namespace {

int check_cfg(const pmc_chunk_cfg* c) {
  if (!c) return fail(PMC_ERR_INVALID, "cfg is NULL");
  if (c->layers < 1 || c->hidden < 1 || c->heads < 1 || c->ffn < 1 || c->seq < 1 || c->microbatch < 1)
    return fail(PMC_ERR_INVALID, "cfg: all sizes must be positive");
  if (c->dtype != PMC_F32 && c->dtype != PMC_BF16) return fail(PMC_ERR_INVALID, "cfg: dtype %d", c->dtype);
  if (c->hidden % c->heads) return fail(PMC_ERR_INVALID, "cfg: hidden %d not divisible by heads %d", c->hidden, c->heads);
  const int dh = c->hidden / c->heads;
  const int64_t tokens = (int64_t)c->seq * c->microbatch;
  if (tokens > (1 << 24)) return fail(PMC_ERR_INVALID, "cfg: too many tokens");
  if (c->dtype == PMC_BF16) {
    if (c->hidden % 8 || c->ffn % 8 || tokens % 8)
      return fail(PMC_ERR_INVALID, "cfg: bf16 mode needs hidden, ffn and tokens to be multiples of 8");
    if (dh > 128) return fail(PMC_ERR_INVALID, "cfg: head size %d > 128", dh);
    if (c->hidden > 12288) return fail(PMC_ERR_INVALID, "cfg: bf16 mode supports hidden <= 12288");
    // the matrix-core attention kernels address one sequence's q|k|v rows inside a 2 GB window
    if (dh % 8 == 0 && (int64_t)c->seq * 3 * c->hidden * 2 > 0x7fffffffLL)
      return fail(PMC_ERR_INVALID, "cfg: seq %d x 3 x hidden %d in bf16 exceeds 2 GB per sequence", c->seq, c->hidden);
  } else {
    if (c->hidden % 4 || c->ffn % 4 || tokens % 4)
      return fail(PMC_ERR_INVALID, "cfg: fp32 mode needs hidden, ffn and tokens to be multiples of 4");
    if (dh > 128) return fail(PMC_ERR_INVALID, "cfg: head size %d > 128", dh);
    if (c->hidden > 4096) return fail(PMC_ERR_INVALID, "cfg: fp32 mode supports hidden <= 4096");
  }
  if (!(c->ln_eps >= 0.f)) return fail(PMC_ERR_INVALID, "cfg: ln_eps must be >= 0");
  return PMC_OK;
}

size_t esize(const pmc_chunk_cfg& c) { return c.dtype == PMC_F32 ? 4 : 2; }

size_t unit_bytes_of(const pmc_chunk_cfg& c) {
  const size_t t = (size_t)c.seq * c.microbatch;
  return (size_t)c.layers * ((size_t)(8 * (size_t)c.hidden + 2 * (size_t)c.ffn) * t * esize(c) + (size_t)(4 + c.heads) * t * 4);
}
size_t stats_bytes_of(const pmc_chunk_cfg& c) {
  return (size_t)c.layers * (size_t)(4 + c.heads) * c.seq * c.microbatch * 4;
}

WorkspaceLayout workspace_of(const pmc_chunk_cfg& c) {
  const int t = c.seq * c.microbatch;
  const size_t e = esize(c);
  WorkspaceLayout w;
  size_t at = 0;
  w.t_h = at;
  at += align256((size_t)t * c.hidden * e);
  w.attn = at;
  at += k::attention_backward_scratch_bytes(c.dtype, c.microbatch, c.seq, c.heads, c.hidden / c.heads);
  w.partial = at;
  // one region per LayerNorm of the backward pass (their reductions are run together at its end)
  const size_t pf = k::layernorm_backward_scratch_floats(t, c.hidden);
  w.partial_stride = align256(pf * sizeof(float));
  at += w.partial_stride * (size_t)std::min(2 * c.layers, (int)k::LnPartialJobs::kMax);
  // split-K partial products of the skinny projections (F and B write [tokens, hidden] outputs)
  size_t g = 0;
  const int h = c.hidden, f = c.ffn;
  const int shapes[7][3] = {{t, 3 * h, h}, {t, h, h}, {t, f, h}, {t, h, f}, {t, h, 3 * h}, {f, h, t}, {h, 3 * h, t}};
  for (const auto& sh : shapes) g = std::max(g, k::gemm_scratch_bytes(c.dtype, sh[0], sh[1], sh[2]));
  w.gemm = at;
  w.gemm_bytes = g;
  at += align256(g);
  w.total = at;
  return w;
}

#define PMC_TRY(expr)          \
  do {                         \
    int rc_ = (expr);          \
    if (rc_ != PMC_OK) return rc_; \
  } while (0)

// Runs `call` (which enqueues one operation) between two events when tracing is on.
template <typename F>
int traced(pmc_ctx* ctx, int op, int pass, int m, int n, int k, int variant, F&& call) {
  if (!ctx->tracing || ctx->trace.size() >= ctx->trace_capacity) return call();
  TraceSlot t;
  t.rec = pmc_trace_rec{op, pass, m, n, k, variant, 0.f};
  if (hipEventCreate(&t.e0) != hipSuccess || hipEventCreate(&t.e1) != hipSuccess)
    return fail(PMC_ERR_HIP, "trace: cannot create events");
  (void)hipEventRecord(t.e0, ctx->stream);
  const int rc = call();
  (void)hipEventRecord(t.e1, ctx->stream);
  ctx->trace.push_back(t);
  return rc;
}

int t_gemm(pmc_ctx* ctx, int pass, k::GemmArgs g, const WorkspaceLayout& wsl) {
  if (wsl.gemm_bytes) {
    g.ws = ctx->ws + wsl.gemm;
    g.ws_bytes = wsl.gemm_bytes;
  }
  const int variant = (g.trans_a ? 1 : 0) | (g.trans_b ? 2 : 0) | (g.epilogue << 2);
  return traced(ctx, PMC_OP_GEMM, pass, g.M, g.N, g.K, variant, [&] { return k::gemm(ctx->stream, g); });
}

const void* P(const pmc_chunk* ch, int layer, int idx) { return ch->params[(size_t)layer * PMC_PARAMS_PER_LAYER + idx]; }
float* G(const pmc_chunk* ch, int layer, int idx) { return ch->grads[(size_t)layer * PMC_PARAMS_PER_LAYER + idx]; }
enum { LN1_G, LN1_B, W_QKV, B_QKV, W_O, B_O, LN2_G, LN2_B, W_1, B_1, W_2, B_2 };

int ready(const pmc_chunk* ch, const char* what) {
  if (!ch) return fail(PMC_ERR_INVALID, "%s: chunk is NULL", what);
  if (!ch->bound) return fail(PMC_ERR_STATE, "%s: parameters are not bound", what);
  const pmc_ctx* ctx = ch->ctx;
  if (!ctx->pool.base) return fail(PMC_ERR_STATE, "%s: no activation pool attached", what);
  if (ctx->pool.slab_bytes < ch->unit_bytes)
    return fail(PMC_ERR_NOMEM, "%s: pool slabs of %zu bytes cannot hold a unit of %zu bytes", what, ctx->pool.slab_bytes,
                ch->unit_bytes);
  if (!ctx->ws || ctx->ws_bytes < ch->wsl.total)
    return fail(PMC_ERR_NOMEM, "%s: workspace of %zu bytes, pass needs %zu", what, ctx->ws_bytes, ch->wsl.total);
  return PMC_OK;
}

k::GemmArgs gemm_args(const pmc_chunk* ch, bool ta, bool tb, int M, int N, int K, const void* A, int lda, const void* B,
                      int ldb, void* C, int ldc, int epi, const void* bias = nullptr, const void* resid = nullptr,
                      void* aux = nullptr) {
  k::GemmArgs g;
  g.dtype = ch->cfg.dtype;
  g.trans_a = ta; g.trans_b = tb;
  g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.epilogue = epi; g.bias = bias; g.resid = resid; g.aux = aux;
  return g;
}

}  // namespace

int chunk_release(pmc_chunk* ch, int32_t mb);

// Takes the slab for (chunk, mb) without running anything (1F1B: a stage takes both its chunks'
// units when its F starts).
int chunk_reserve(pmc_chunk* ch, int32_t mb, int device) {
  PMC_TRY(ready(ch, "reserve"));
  if (ch->live.count(mb)) return fail(PMC_ERR_STATE, "microbatch %d is already live in this chunk", mb);
  void* slab = ch->ctx->pool.take(device, (int64_t)ch->unit_bytes);
  if (!slab) return fail(PMC_ERR_NOMEM, "activation pool exhausted (%lld slabs in use)", (long long)ch->ctx->pool.live);
  Micro m;
  m.slab = (char*)slab;
  m.state = kReserved;
  m.device = device;
  ch->live[mb] = m;
  return PMC_OK;
}

int chunk_forward(pmc_chunk* ch, int32_t mb, const void* x, void* y, int device) {
  PMC_TRY(ready(ch, "stage_forward"));
  if (!x || !y) return fail(PMC_ERR_INVALID, "stage_forward: NULL tensor");
  auto it = ch->live.find(mb);
  if (it != ch->live.end() && it->second.state != kReserved)
    return fail(PMC_ERR_STATE, "stage_forward: microbatch %d is already live in this chunk", mb);
  bool reserved_here = false;
  if (it == ch->live.end()) {
    PMC_TRY(chunk_reserve(ch, mb, device));
    it = ch->live.find(mb);
    reserved_here = true;
  }
  Micro& m = it->second;
  const pmc_chunk_cfg& c = ch->cfg;
  hipStream_t st = ch->ctx->stream;
  const int T = ch->tokens, h = c.hidden, f = c.ffn, L = c.layers;
  auto layers = [&]() -> int {
  for (int l = 0; l < L; ++l) {
    const LayerOffsets& o = ch->off[l];
    char* s = m.slab;
    const void* xin = l == 0 ? x : (const void*)(s + o.x);
    PMC_TRY(traced(ch->ctx, PMC_OP_LN_FWD, PMC_F, T, h, 0, 0, [&] { return k::layernorm_forward(st, c.dtype, T, h, xin, P(ch, l, LN1_G), P(ch, l, LN1_B), c.ln_eps, s + o.a,
                                 (float*)(s + o.mean1), (float*)(s + o.rstd1), l == 0 ? s + o.x : nullptr); }));
    PMC_TRY(t_gemm(ch->ctx, PMC_F, gemm_args(ch, false, false, T, 3 * h, h, s + o.a, h, P(ch, l, W_QKV), 3 * h, s + o.qkv, 3 * h,
                                  PMC_EPI_BIAS, P(ch, l, B_QKV)), ch->wsl));
    PMC_TRY(traced(ch->ctx, PMC_OP_ATTN_FWD, PMC_F, T, c.heads, ch->head_dim, 0, [&] { return k::attention_forward(st, c.dtype, c.microbatch, c.seq, c.heads, ch->head_dim, c.causal, s + o.qkv, s + o.o,
                                 (float*)(s + o.lse)); }));
    PMC_TRY(t_gemm(ch->ctx, PMC_F, gemm_args(ch, false, false, T, h, h, s + o.o, h, P(ch, l, W_O), h, s + o.xmid, h,
                                  PMC_EPI_BIAS_RESID, P(ch, l, B_O), s + o.x), ch->wsl));
    PMC_TRY(traced(ch->ctx, PMC_OP_LN_FWD, PMC_F, T, h, 0, 0, [&] { return k::layernorm_forward(st, c.dtype, T, h, s + o.xmid, P(ch, l, LN2_G), P(ch, l, LN2_B), c.ln_eps, s + o.c,
                                 (float*)(s + o.mean2), (float*)(s + o.rstd2), nullptr); }));
    // FC1: the slab keeps gelu(u) for FC2 and W, and gelu'(u) (in the slot called u) for B
    PMC_TRY(t_gemm(ch->ctx, PMC_F, gemm_args(ch, false, false, T, f, h, s + o.c, h, P(ch, l, W_1), f, s + o.u, f, PMC_EPI_BIAS_GELU_GRAD,
                                  P(ch, l, B_1), nullptr, s + o.g), ch->wsl));
    void* out = l == L - 1 ? y : (void*)(s + ch->off[l + 1].x);
    PMC_TRY(t_gemm(ch->ctx, PMC_F, gemm_args(ch, false, false, T, h, f, s + o.g, f, P(ch, l, W_2), h, out, h, PMC_EPI_BIAS_RESID,
                                  P(ch, l, B_2), s + o.xmid), ch->wsl));
  }
  return PMC_OK;
  };
  const int rc = layers();
  if (rc != PMC_OK) {
    // a launch failed part-way: the unit this call took goes back to the pool (kernels already
    // enqueued only write inside the slab, which nothing else uses before they have run: the stream
    // orders them); a unit reserved earlier by the replayer stays reserved for the replayer to return
    if (reserved_here) (void)chunk_release(ch, mb);
    return rc;
  }
  m.state = kForwardDone;
  return PMC_OK;
}

int chunk_backward_input(pmc_chunk* ch, int32_t mb, const void* dy, void* dx) {
  PMC_TRY(ready(ch, "stage_backward_input"));
  if (!dy || !dx) return fail(PMC_ERR_INVALID, "stage_backward_input: NULL tensor");
  auto it = ch->live.find(mb);
  if (it == ch->live.end() || it->second.state == kReserved)
    return fail(PMC_ERR_STATE, "stage_backward_input: microbatch %d has no forward pass in this chunk", mb);
  if (it->second.state != kForwardDone)
    return fail(PMC_ERR_STATE, "stage_backward_input: microbatch %d already had its backward pass", mb);
  Micro& m = it->second;
  const pmc_chunk_cfg& c = ch->cfg;
  hipStream_t st = ch->ctx->stream;
  const int T = ch->tokens, h = c.hidden, f = c.ffn, L = c.layers;
  char* s = m.slab;
  char* ws = ch->ctx->ws;
  void* t_h = ws + ch->wsl.t_h;
  void* attn_ws = ws + ch->wsl.attn;
  // LayerNorm gain/bias gradients: each call leaves its partial sums in a region of its own and
  // one launch adds them all up (when the regions run out, and at the end of the pass)
  k::LnPartialJobs ln_jobs;
  auto next_partial = [&]() { return (float*)(ws + ch->wsl.partial + (size_t)ln_jobs.count * ch->wsl.partial_stride); };
  auto flush_ln = [&](bool force) {
    if (ln_jobs.count == 0 || (!force && ln_jobs.count < k::LnPartialJobs::kMax)) return (int)PMC_OK;
    const int rc = traced(ch->ctx, PMC_OP_LN_BWD, PMC_B, ln_jobs.count, 2 * h, 0, 1, [&] { return k::layernorm_backward_reduce(st, h, ln_jobs); });
    ln_jobs.count = 0;
    return rc;
  };
  for (int l = L - 1; l >= 0; --l) {
    const LayerOffsets& o = ch->off[l];
    const void* dyl = l == L - 1 ? dy : (const void*)(s + ch->off[l + 1].x);
    // dU = (dY . W2^T) * gelu'(U), written over the gelu'(U) that F left
    PMC_TRY(t_gemm(ch->ctx, PMC_B, gemm_args(ch, false, true, T, f, h, dyl, h, P(ch, l, W_2), h, s + o.u, f, PMC_EPI_MUL, nullptr,
                                  nullptr, s + o.u), ch->wsl));
    // dC = dU . W1^T
    PMC_TRY(t_gemm(ch->ctx, PMC_B, gemm_args(ch, false, true, T, h, f, s + o.u, f, P(ch, l, W_1), f, t_h, h, PMC_EPI_NONE), ch->wsl));
    // dX_mid = dY + LN2 input-gradient(dC), written over X_mid; LN2 gain/bias gradients
    PMC_TRY(traced(ch->ctx, PMC_OP_LN_BWD, PMC_B, T, h, 0, 0, [&] { return k::layernorm_backward(st, c.dtype, T, h, t_h, s + o.xmid, P(ch, l, LN2_G), (const float*)(s + o.mean2),
                                  (const float*)(s + o.rstd2), dyl, s + o.xmid, G(ch, l, LN2_G), G(ch, l, LN2_B), next_partial(), &ln_jobs); }));
    PMC_TRY(flush_ln(false));
    // dO = dX_mid . Wo^T
    PMC_TRY(t_gemm(ch->ctx, PMC_B, gemm_args(ch, false, true, T, h, h, s + o.xmid, h, P(ch, l, W_O), h, t_h, h, PMC_EPI_NONE), ch->wsl));
    // dQKV, written over QKV
    PMC_TRY(traced(ch->ctx, PMC_OP_ATTN_BWD, PMC_B, T, c.heads, ch->head_dim, 0, [&] { return k::attention_backward(st, c.dtype, c.microbatch, c.seq, c.heads, ch->head_dim, c.causal, s + o.qkv, s + o.o,
                                  (const float*)(s + o.lse), t_h, s + o.qkv, attn_ws); }));
    // dA = dQKV . Wqkv^T
    PMC_TRY(t_gemm(ch->ctx, PMC_B, gemm_args(ch, false, true, T, h, 3 * h, s + o.qkv, 3 * h, P(ch, l, W_QKV), 3 * h, t_h, h,
                                  PMC_EPI_NONE), ch->wsl));
    // dX = dX_mid + LN1 input-gradient(dA): over X for inner layers, to the caller for layer 0
    void* out = l == 0 ? dx : (void*)(s + o.x);
    PMC_TRY(traced(ch->ctx, PMC_OP_LN_BWD, PMC_B, T, h, 0, 0, [&] { return k::layernorm_backward(st, c.dtype, T, h, t_h, s + o.x, P(ch, l, LN1_G), (const float*)(s + o.mean1),
                                  (const float*)(s + o.rstd1), s + o.xmid, out, G(ch, l, LN1_G), G(ch, l, LN1_B), next_partial(), &ln_jobs); }));
    PMC_TRY(flush_ln(false));
  }
  PMC_TRY(flush_ln(true));
  // keep the chunk's dY for W of the top layer in the slot of the (now dead) chunk input
  PMC_TRY(traced(ch->ctx, PMC_OP_COPY, PMC_B, T, h, 0, 0, [&] { return k::copy_rows(st, c.dtype, T, h, dy, h, s + ch->off[0].x, h); }));
  m.state = kBackwardDone;
  ch->ctx->pool.shrink(m.device, (int64_t)ch->stats_bytes);
  return PMC_OK;
}

// The weight-gradient products of a pass do not depend on each other.  Every second one goes to a
// second stream (fork and join with events inside the pass): workgroups of two different products
// then share the chip, one product's read-modify-write of dW overlaps the other's matrix work, the
// tail of one fills with the head of the next, and the memory-bound bias-gradient sums run under a
// product (measured on the W pass: -5 % at hidden 2048 / 1024 tokens, -6 % at 4096 / 2048, -5 % at
// 5120 / 4096; a third and fourth stream gain nothing more).  The w_streams tuning switch forces the choice.
// Off while tracing, whose per-operation events assume one stream.
int w_pass_streams(const pmc_chunk* ch) {
  if (ch->ctx->tracing || ch->cfg.dtype != PMC_BF16) return 1;
  if (const int f = tuning(kTuneWStreams); f >= 0) return f;
  return 2;
}

int side_streams(pmc_ctx* ctx, int n) {
  if (!ctx->fork && hipEventCreateWithFlags(&ctx->fork, hipEventDisableTiming) != hipSuccess)
    return fail(PMC_ERR_HIP, "cannot create the fork event of the W pass");
  for (int i = 0; i < n; ++i) {
    if (ctx->side[i]) continue;
    if (hipStreamCreateWithFlags(&ctx->side[i], hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->join[i], hipEventDisableTiming) != hipSuccess)
      return fail(PMC_ERR_HIP, "cannot create a side stream of the W pass");
  }
  return PMC_OK;
}

// Makes the context's stream wait for the first n side streams.  `rc` is what the forked work
// returned: a failure there is reported in preference to one here; if the join itself cannot be
// enqueued the side streams are drained on the host instead.
int join_side_streams(pmc_ctx* ctx, int n, int rc) {
  bool ok = true;
  for (int i = 0; i < n; ++i)
    if (hipEventRecord(ctx->join[i], ctx->side[i]) != hipSuccess || hipStreamWaitEvent(ctx->stream, ctx->join[i], 0) != hipSuccess) {
      ok = false;
      (void)hipStreamSynchronize(ctx->side[i]);
    }
  if (rc != PMC_OK) return rc;
  return ok ? (int)PMC_OK : fail(PMC_ERR_HIP, "stage_backward_weight: cannot join a side stream");
}

int chunk_backward_weight_one(pmc_chunk* ch, int32_t mb, bool release) {
  auto it = ch->live.find(mb);
  if (it == ch->live.end() || it->second.state != kBackwardDone)
    return fail(PMC_ERR_STATE, "stage_backward_weight: microbatch %d has not had its backward-input pass", mb);
  Micro& m = it->second;
  const pmc_chunk_cfg& c = ch->cfg;
  pmc_ctx* ctx = ch->ctx;
  hipStream_t st = ctx->stream;
  const int T = ch->tokens, h = c.hidden, f = c.ffn, L = c.layers;
  char* s = m.slab;
  const int ns = w_pass_streams(ch);
  const bool two = ns > 1;
  if (two) {
    PMC_TRY(side_streams(ctx, ns - 1));
    if (hipEventRecord(ctx->fork, st) != hipSuccess) return fail(PMC_ERR_HIP, "stage_backward_weight: cannot fork");
    for (int i = 0; i < ns - 1; ++i)
      if (hipStreamWaitEvent(ctx->side[i], ctx->fork, 0) != hipSuccess)
        return fail(PMC_ERR_HIP, "stage_backward_weight: cannot fork a side stream");
  }
  // product number `slot` of the pass: stream slot % ns (0 = the caller's); side streams get no
  // split-K scratch (the first stream's products own it)
  int slot = 0;
  auto side_gemm = [&](k::GemmArgs g) {
    const int which = slot++ % ns;
    if (which == 0) return t_gemm(ctx, PMC_W, g, ch->wsl);
    g.ws = nullptr;
    g.ws_bytes = 0;
    return k::gemm(ctx->side[which - 1], g);
  };
  auto products = [&]() -> int {
    for (int l = L - 1; l >= 0; --l) {
      const LayerOffsets& o = ch->off[l];
      const void* dxout = s + (l == L - 1 ? ch->off[0].x : ch->off[l + 1].x);
      // the four bias gradients of the layer in one launch
      k::ColumnSumJobs jobs = {};
      jobs.count = 4;
      const void* src[4] = {dxout, s + o.u, s + o.xmid, s + o.qkv};
      const int width[4] = {h, f, h, 3 * h};
      const int which[4] = {B_2, B_1, B_O, B_QKV};
      for (int j = 0; j < 4; ++j) {
        jobs.a[j] = src[j];
        jobs.out[j] = G(ch, l, which[j]);
        jobs.n[j] = jobs.lda[j] = width[j];
      }
      // (memory-bound, no matrix work: on the second stream it runs under the first product)
      PMC_TRY(traced(ctx, PMC_OP_COLSUM, PMC_W, T, 0, 0, 0, [&] { return k::column_sums(two ? ctx->side[ns - 2] : st, c.dtype, T, jobs); }));
      PMC_TRY(side_gemm(gemm_args(ch, true, false, f, h, T, s + o.g, f, dxout, h, G(ch, l, W_2), h, PMC_EPI_ACCUM_F32)));
      PMC_TRY(side_gemm(gemm_args(ch, true, false, h, f, T, s + o.c, h, s + o.u, f, G(ch, l, W_1), f, PMC_EPI_ACCUM_F32)));
      PMC_TRY(side_gemm(gemm_args(ch, true, false, h, h, T, s + o.o, h, s + o.xmid, h, G(ch, l, W_O), h, PMC_EPI_ACCUM_F32)));
      PMC_TRY(side_gemm(gemm_args(ch, true, false, h, 3 * h, T, s + o.a, h, s + o.qkv, 3 * h, G(ch, l, W_QKV), 3 * h,
                                  PMC_EPI_ACCUM_F32)));
    }
    return PMC_OK;
  };
  // whatever happened in between, the caller's stream waits for the side stream: a failed pass must
  // not leave work on it that still reads the slab or writes the gradients
  const int rc = products();
  PMC_TRY(join_side_streams(ctx, ns - 1, rc));
  if (release) {
    ch->ctx->pool.give(m.slab, m.device, (int64_t)(ch->unit_bytes - ch->stats_bytes));
    ch->live.erase(it);
  }
  return PMC_OK;
}

// W of 2 .. PMC_MAX_QUEUED_W microbatches of a bf16 chunk at once: per layer, the bias gradients of
// each microbatch, then every weight gradient as one product over the microbatches' concatenated
// token axis (one read-modify-write of the fp32 accumulator for the whole group).
int chunk_backward_weight_group(pmc_chunk* ch, const int32_t* mbs, int count) {
  const pmc_chunk_cfg& c = ch->cfg;
  pmc_ctx* ctx = ch->ctx;
  hipStream_t st = ctx->stream;
  const int T = ch->tokens, h = c.hidden, f = c.ffn, L = c.layers;
  char* slab[PMC_MAX_QUEUED_W];
  for (int i = 0; i < count; ++i) slab[i] = ch->live.find(mbs[i])->second.slab;
  const int ns = w_pass_streams(ch);  // as in the single-microbatch pass: every second product on a second stream
  if (ns > 1) {
    PMC_TRY(side_streams(ctx, 1));
    if (hipEventRecord(ctx->fork, st) != hipSuccess || hipStreamWaitEvent(ctx->side[0], ctx->fork, 0) != hipSuccess)
      return fail(PMC_ERR_HIP, "stage_backward_weight: cannot fork the second stream");
  }
  int slot = 0;
  auto grouped = [&](int M, int N, auto a_of, int lda, auto b_of, int ldb, float* C) {
    hipStream_t on = (ns > 1 && (slot++ & 1)) ? ctx->side[0] : st;
    k::GroupedWgradArgs g;
    g.M = M; g.N = N; g.K = T; g.count = count; g.lda = lda; g.ldb = ldb; g.C = C; g.ldc = N;
    for (int i = 0; i < count; ++i) {
      g.A[i] = a_of(slab[i]);
      g.B[i] = b_of(slab[i]);
    }
    const int variant = 1 | (PMC_EPI_ACCUM_F32 << 2);
    return traced(ctx, PMC_OP_GEMM, PMC_W, M, N, T * count, variant, [&] { return k::gemm_bf16_grouped_wgrad(on, g); });
  };
  auto products = [&]() -> int {
    for (int l = L - 1; l >= 0; --l) {
      const LayerOffsets& o = ch->off[l];
      const size_t dxout_off = l == L - 1 ? ch->off[0].x : ch->off[l + 1].x;
      for (int i = 0; i < count; ++i) {
        char* s = slab[i];
        k::ColumnSumJobs jobs = {};
        jobs.count = 4;
        const void* src[4] = {s + dxout_off, s + o.u, s + o.xmid, s + o.qkv};
        const int width[4] = {h, f, h, 3 * h};
        const int which[4] = {B_2, B_1, B_O, B_QKV};
        for (int j = 0; j < 4; ++j) {
          jobs.a[j] = src[j];
          jobs.out[j] = G(ch, l, which[j]);
          jobs.n[j] = jobs.lda[j] = width[j];
        }
        PMC_TRY(traced(ctx, PMC_OP_COLSUM, PMC_W, T, 0, 0, 0, [&] { return k::column_sums(ns > 1 ? ctx->side[0] : st, c.dtype, T, jobs); }));
      }
      PMC_TRY(grouped(f, h, [&](char* s) { return s + o.g; }, f, [&](char* s) { return s + dxout_off; }, h, G(ch, l, W_2)));
      PMC_TRY(grouped(h, f, [&](char* s) { return s + o.c; }, h, [&](char* s) { return s + o.u; }, f, G(ch, l, W_1)));
      PMC_TRY(grouped(h, h, [&](char* s) { return s + o.o; }, h, [&](char* s) { return s + o.xmid; }, h, G(ch, l, W_O)));
      PMC_TRY(grouped(h, 3 * h, [&](char* s) { return s + o.a; }, h, [&](char* s) { return s + o.qkv; }, 3 * h, G(ch, l, W_QKV)));
    }
    return PMC_OK;
  };
  const int rc = products();
  PMC_TRY(join_side_streams(ctx, ns > 1 ? 1 : 0, rc));
  for (int i = 0; i < count; ++i) {
    auto it = ch->live.find(mbs[i]);
    ctx->pool.give(it->second.slab, it->second.device, (int64_t)(ch->unit_bytes - ch->stats_bytes));
    ch->live.erase(it);
  }
  return PMC_OK;
}

// Returns a slab whose W has run with release = false.
int chunk_release(pmc_chunk* ch, int32_t mb) {
  auto it = ch->live.find(mb);
  if (it == ch->live.end()) return fail(PMC_ERR_STATE, "release: microbatch %d is not live", mb);
  Micro& m = it->second;
  const int64_t rest = m.state == kBackwardDone ? (int64_t)(ch->unit_bytes - ch->stats_bytes) : (int64_t)ch->unit_bytes;
  ch->ctx->pool.give(m.slab, m.device, rest);
  ch->live.erase(it);
  return PMC_OK;
}

// Returns every live slab of the chunk, whatever its state (after a failed replay).
void chunk_release_all(pmc_chunk* ch) {
  while (!ch->live.empty()) (void)chunk_release(ch, ch->live.begin()->first);
}

size_t chunk_unit_bytes(const pmc_chunk* ch) { return ch->unit_bytes; }
size_t chunk_stats_bytes(const pmc_chunk* ch) { return ch->stats_bytes; }
size_t chunk_workspace_bytes(const pmc_chunk* ch) { return ch->wsl.total; }
pmc_ctx* chunk_ctx(const pmc_chunk* ch) { return ch->ctx; }
const pmc_chunk_cfg& chunk_cfg(const pmc_chunk* ch) { return ch->cfg; }
hipStream_t ctx_stream(const pmc_ctx* ctx) { return ctx->stream; }
char* ctx_workspace(const pmc_ctx* ctx, size_t* bytes) {
  *bytes = ctx->ws_bytes;
  return ctx->ws;
}
void ctx_device_peaks(pmc_ctx* ctx, int d, int64_t unit_bytes, pmc_device_peak* out) {
  for (int i = 0; i < d; ++i) {
    const Pool::Dev& dv = ctx->pool.dev[i];
    out[i].peak_live_units = dv.peak_units;
    out[i].peak_live_bytes = dv.peak_units * unit_bytes;
    out[i].peak_tensor_bytes = dv.peak_tensor_bytes;
  }
}

}  // namespace pmc

using namespace pmc;

extern "C" {

int pmc_create(void* hip_stream, pmc_ctx** out) {
  if (!out) return fail(PMC_ERR_INVALID, "out is NULL");
  auto* ctx = new (std::nothrow) pmc_ctx;
  if (!ctx) return fail(PMC_ERR_NOMEM, "host allocation failed");
  ctx->stream = (hipStream_t)hip_stream;
  *out = ctx;
  return PMC_OK;
}

void pmc_destroy(pmc_ctx* ctx) { delete ctx; }

int pmc_pool_attach(pmc_ctx* ctx, void* arena, size_t bytes, size_t slab_bytes) {
  if (!ctx || !arena) return fail(PMC_ERR_INVALID, "pool_attach: NULL argument");
  if ((uintptr_t)arena & 255) return fail(PMC_ERR_INVALID, "pool_attach: arena must be 256-byte aligned");
  if (slab_bytes == 0) return fail(PMC_ERR_INVALID, "pool_attach: slab_bytes is 0");
  if (ctx->pool.live) return fail(PMC_ERR_STATE, "pool_attach: %lld slabs still in use", (long long)ctx->pool.live);
  const size_t sb = align256(slab_bytes);
  const int64_t n = (int64_t)(bytes / sb);
  if (n < 1) return fail(PMC_ERR_NOMEM, "pool_attach: arena of %zu bytes holds no slab of %zu bytes", bytes, sb);
  ctx->pool = Pool();
  ctx->pool.base = (char*)arena;
  ctx->pool.slab_bytes = sb;
  ctx->pool.slabs = n;
  for (int64_t i = 0; i < n; ++i) ctx->pool.free_list.insert(i);
  return PMC_OK;
}

int64_t pmc_pool_live_slabs(const pmc_ctx* ctx) { return ctx ? ctx->pool.live : 0; }
int64_t pmc_pool_peak_slabs(const pmc_ctx* ctx) { return ctx ? ctx->pool.peak : 0; }
void pmc_pool_reset_peak(pmc_ctx* ctx) {
  if (ctx) ctx->pool.reset_peaks();
}

int pmc_workspace_attach(pmc_ctx* ctx, void* workspace, size_t bytes) {
  if (!ctx || !workspace) return fail(PMC_ERR_INVALID, "workspace_attach: NULL argument");
  if ((uintptr_t)workspace & 255) return fail(PMC_ERR_INVALID, "workspace_attach: must be 256-byte aligned");
  ctx->ws = (char*)workspace;
  ctx->ws_bytes = bytes;
  return PMC_OK;
}

size_t pmc_activation_bytes(const pmc_chunk_cfg* cfg) { return check_cfg(cfg) == PMC_OK ? unit_bytes_of(*cfg) : 0; }
size_t pmc_activation_stats_bytes(const pmc_chunk_cfg* cfg) { return check_cfg(cfg) == PMC_OK ? stats_bytes_of(*cfg) : 0; }
size_t pmc_pass_workspace_bytes(const pmc_chunk_cfg* cfg) { return check_cfg(cfg) == PMC_OK ? workspace_of(*cfg).total : 0; }

int pmc_chunk_create(pmc_ctx* ctx, const pmc_chunk_cfg* cfg, pmc_chunk** out) {
  if (!ctx || !out) return fail(PMC_ERR_INVALID, "chunk_create: NULL argument");
  PMC_TRY(check_cfg(cfg));
  auto* ch = new (std::nothrow) pmc_chunk;
  if (!ch) return fail(PMC_ERR_NOMEM, "host allocation failed");
  ch->ctx = ctx;
  ch->cfg = *cfg;
  ch->tokens = cfg->seq * cfg->microbatch;
  ch->head_dim = cfg->hidden / cfg->heads;
  ch->esz = esize(*cfg);
  ch->unit_bytes = unit_bytes_of(*cfg);
  ch->stats_bytes = stats_bytes_of(*cfg);
  ch->wsl = workspace_of(*cfg);
  const size_t th = (size_t)ch->tokens * cfg->hidden * ch->esz, tf = (size_t)ch->tokens * cfg->ffn * ch->esz;
  const size_t per_layer = 8 * th + 2 * tf;
  const size_t st_layer = (size_t)(4 + cfg->heads) * ch->tokens * 4;
  const size_t stats0 = per_layer * cfg->layers;
  ch->off.resize(cfg->layers);
  for (int l = 0; l < cfg->layers; ++l) {
    LayerOffsets& o = ch->off[l];
    size_t at = per_layer * l;
    o.x = at; at += th;
    o.a = at; at += th;
    o.qkv = at; at += 3 * th;
    o.o = at; at += th;
    o.xmid = at; at += th;
    o.c = at; at += th;
    o.u = at; at += tf;
    o.g = at; at += tf;
    size_t sa = stats0 + st_layer * l;
    const size_t tb = (size_t)ch->tokens * 4;
    o.mean1 = sa; sa += tb;
    o.rstd1 = sa; sa += tb;
    o.mean2 = sa; sa += tb;
    o.rstd2 = sa; sa += tb;
    o.lse = sa;
  }
  ++ctx->chunks_alive;
  *out = ch;
  return PMC_OK;
}

void pmc_chunk_destroy(pmc_chunk* ch) {
  if (!ch) return;
  for (auto& kv : ch->live) {
    const int64_t rest = kv.second.state == kBackwardDone ? (int64_t)(ch->unit_bytes - ch->stats_bytes) : (int64_t)ch->unit_bytes;
    ch->ctx->pool.give(kv.second.slab, kv.second.device, rest);
  }
  --ch->ctx->chunks_alive;
  delete ch;
}

int pmc_chunk_bind(pmc_chunk* ch, const void* const* params, void* const* grads_fp32) {
  if (!ch || !params || !grads_fp32) return fail(PMC_ERR_INVALID, "chunk_bind: NULL argument");
  const size_t n = (size_t)ch->cfg.layers * PMC_PARAMS_PER_LAYER;
  for (size_t i = 0; i < n; ++i) {
    if (!params[i] || !grads_fp32[i]) return fail(PMC_ERR_INVALID, "chunk_bind: pointer %zu is NULL", i);
    if (((uintptr_t)params[i] & 15) || ((uintptr_t)grads_fp32[i] & 15))
      return fail(PMC_ERR_INVALID, "chunk_bind: pointer %zu is not 16-byte aligned", i);
  }
  ch->params.assign(params, params + n);
  ch->grads.resize(n);
  for (size_t i = 0; i < n; ++i) ch->grads[i] = (float*)grads_fp32[i];
  ch->bound = true;
  return PMC_OK;
}

int stage_forward(pmc_chunk* ch, int32_t mb, const void* x, void* y) { return chunk_forward(ch, mb, x, y, 0); }
int stage_forward_on(pmc_chunk* ch, int32_t mb, const void* x, void* y, int32_t device) {
  if (device < 0) return fail(PMC_ERR_INVALID, "stage_forward_on: device %d", device);
  return chunk_forward(ch, mb, x, y, device);
}
int stage_backward_input(pmc_chunk* ch, int32_t mb, const void* dy, void* dx) { return chunk_backward_input(ch, mb, dy, dx); }

int stage_abandon(pmc_chunk* ch, int32_t mb) {
  if (!ch) return fail(PMC_ERR_INVALID, "stage_abandon: chunk is NULL");
  return chunk_release(ch, mb);
}

int stage_backward_weight(pmc_chunk* ch, const int32_t* mbs, int32_t count) {
  PMC_TRY(ready(ch, "stage_backward_weight"));
  if (!mbs || count < 1) return fail(PMC_ERR_INVALID, "stage_backward_weight: empty list");
  for (int32_t i = 0; i < count; ++i) {
    auto it = ch->live.find(mbs[i]);
    if (it == ch->live.end() || it->second.state != kBackwardDone)
      return fail(PMC_ERR_STATE, "stage_backward_weight: microbatch %d has not had its backward-input pass", mbs[i]);
    for (int32_t j = 0; j < i; ++j)
      if (mbs[j] == mbs[i]) return fail(PMC_ERR_INVALID, "stage_backward_weight: microbatch %d listed twice", mbs[i]);
  }
  // bf16 chunks whose token count fills whole 64-wide K tiles: groups of queued microbatches go
  // through one product per weight; everything else one microbatch at a time
  const bool group = ch->cfg.dtype == PMC_BF16 && ch->tokens % 64 == 0;
  for (int32_t i = 0; i < count;) {
    const int32_t n = group ? (count - i < PMC_MAX_QUEUED_W ? count - i : PMC_MAX_QUEUED_W) : 1;
    if (n > 1) PMC_TRY(chunk_backward_weight_group(ch, mbs + i, n));
    else PMC_TRY(chunk_backward_weight_one(ch, mbs[i], true));
    i += n;
  }
  return PMC_OK;
}

/* ---- tracing ---- */

int pmc_trace_begin(pmc_ctx* ctx, int32_t capacity) {
  if (!ctx || capacity < 1) return fail(PMC_ERR_INVALID, "trace_begin: bad argument");
  if (ctx->tracing) return fail(PMC_ERR_STATE, "trace_begin: already tracing");
  ctx->trace.clear();
  ctx->trace.reserve((size_t)capacity);
  ctx->trace_capacity = (size_t)capacity;
  ctx->tracing = true;
  return PMC_OK;
}

int pmc_trace_end(pmc_ctx* ctx, pmc_trace_rec* out, int32_t capacity, int32_t* count) {
  if (!ctx || !out || !count || capacity < 0) return fail(PMC_ERR_INVALID, "trace_end: bad argument");
  if (!ctx->tracing) return fail(PMC_ERR_STATE, "trace_end: not tracing");
  ctx->tracing = false;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  int rc = e == hipSuccess ? PMC_OK : fail(PMC_ERR_HIP, "trace_end: %s", hipGetErrorString(e));
  int32_t n = 0;
  for (TraceSlot& t : ctx->trace) {
    if (rc == PMC_OK && n < capacity) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, t.e0, t.e1) != hipSuccess) ms = -1.f;
      t.rec.ms = ms;
      out[n++] = t.rec;
    }
    (void)hipEventDestroy(t.e0);
    (void)hipEventDestroy(t.e1);
  }
  ctx->trace.clear();
  *count = n;
  return rc;
}

/* ---- single operations ---- */

int pmc_gemm(pmc_ctx* ctx, int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K, const void* A,
             int32_t lda, const void* B, int32_t ldb, void* C, int32_t ldc, int32_t epilogue, const void* bias,
             const void* resid, void* aux) {
  if (!ctx) return fail(PMC_ERR_INVALID, "ctx is NULL");
  k::GemmArgs g;
  g.dtype = dtype; g.trans_a = trans_a != 0; g.trans_b = trans_b != 0;
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.epilogue = epilogue; g.bias = bias; g.resid = resid; g.aux = aux;
  g.ws = ctx->ws; g.ws_bytes = ctx->ws_bytes;
  return k::gemm(ctx->stream, g);
}

int pmc_gemm_grouped_wgrad(pmc_ctx* ctx, int32_t M, int32_t N, int32_t K, int32_t count, const void* const* a, int32_t lda,
                           const void* const* b, int32_t ldb, float* C, int32_t ldc) {
  if (!ctx || !a || !b || !C) return fail(PMC_ERR_INVALID, "pmc_gemm_grouped_wgrad: NULL argument");
  if (count < 1 || count > PMC_MAX_QUEUED_W) return fail(PMC_ERR_INVALID, "pmc_gemm_grouped_wgrad: count %d (1..%d)", count, PMC_MAX_QUEUED_W);
  k::GroupedWgradArgs g;
  g.M = M; g.N = N; g.K = K; g.count = count; g.lda = lda; g.ldb = ldb; g.C = C; g.ldc = ldc;
  for (int i = 0; i < count; ++i) {
    g.A[i] = a[i];
    g.B[i] = b[i];
  }
  return k::gemm_bf16_grouped_wgrad(ctx->stream, g);
}

int pmc_layernorm_forward(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t h, const void* x, const void* gain,
                          const void* bias, float eps, void* y, float* mean, float* rstd, void* x_copy) {
  if (!ctx) return fail(PMC_ERR_INVALID, "ctx is NULL");
  return k::layernorm_forward(ctx->stream, dtype, rows, h, x, gain, bias, eps, y, mean, rstd, x_copy);
}

int pmc_layernorm_backward(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t h, const void* dy, const void* x,
                           const void* gain, const float* mean, const float* rstd, const void* resid, void* dx,
                           float* dgain, float* dbias) {
  if (!ctx) return fail(PMC_ERR_INVALID, "ctx is NULL");
  if (rows <= 0 || h <= 0) return fail(PMC_ERR_INVALID, "layernorm_backward: rows=%d h=%d", rows, h);
  const size_t need = k::layernorm_backward_scratch_floats(rows, h) * sizeof(float);
  if (!ctx->ws || ctx->ws_bytes < need) return fail(PMC_ERR_NOMEM, "layernorm_backward: workspace needs %zu bytes", need);
  return k::layernorm_backward(ctx->stream, dtype, rows, h, dy, x, gain, mean, rstd, resid, dx, dgain, dbias, (float*)ctx->ws);
}

int pmc_layernorm_backward_static(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t h, const void* dy, const void* x,
                                  const void* gain, const float* mean, const float* rstd, const void* resid, void* dx,
                                  float* dgain, float* dbias) {
  if (!ctx) return fail(PMC_ERR_INVALID, "ctx is NULL");
  return k::layernorm_backward_static(ctx->stream, dtype, rows, h, dy, x, gain, mean, rstd, resid, dx, dgain, dbias);
}

int pmc_attention_forward(pmc_ctx* ctx, int32_t dtype, int32_t batch, int32_t seq, int32_t heads, int32_t head_dim,
                          int32_t causal, const void* qkv, void* o, float* lse) {
  if (!ctx) return fail(PMC_ERR_INVALID, "ctx is NULL");
  return k::attention_forward(ctx->stream, dtype, batch, seq, heads, head_dim, causal, qkv, o, lse);
}

int pmc_attention_backward(pmc_ctx* ctx, int32_t dtype, int32_t batch, int32_t seq, int32_t heads, int32_t head_dim,
                           int32_t causal, const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv) {
  if (!ctx) return fail(PMC_ERR_INVALID, "ctx is NULL");
  if (batch <= 0 || seq <= 0 || heads <= 0 || head_dim <= 0) return fail(PMC_ERR_INVALID, "attention_backward: bad shape");
  const size_t need = k::attention_backward_scratch_bytes(dtype, batch, seq, heads, head_dim);
  if (!ctx->ws || ctx->ws_bytes < need) return fail(PMC_ERR_NOMEM, "attention_backward: workspace needs %zu bytes", need);
  return k::attention_backward(ctx->stream, dtype, batch, seq, heads, head_dim, causal, qkv, o, lse, d_o, dqkv, ctx->ws);
}

int pmc_column_sum(pmc_ctx* ctx, int32_t dtype, int32_t rows, int32_t n, const void* a, int32_t lda, float* out) {
  if (!ctx) return fail(PMC_ERR_INVALID, "ctx is NULL");
  if (rows <= 0 || n <= 0) return fail(PMC_ERR_INVALID, "column_sum: rows=%d n=%d", rows, n);
  return k::column_sum(ctx->stream, dtype, rows, n, a, lda, out);
}

}  // extern "C"
