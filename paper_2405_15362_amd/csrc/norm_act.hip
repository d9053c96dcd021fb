// Row-wise kernels bounded by HBM bandwidth: LayerNorm forward, LayerNorm input-gradient (with the
// gain/bias gradient partial sums), column sums for the bias gradients, and a pitched row copy.
// Forward: one 64-lane wave owns a row and the row reductions are wave shuffles.  Backward: one to
// eight waves share a row.  Reductions across rows go through fixed-order partial sums, so results
// do not depend on scheduling.
#include <mutex>

#include "dev_common.h"
#include "kernels.h"

namespace pmc {
namespace k {
namespace {

// Scratch of layernorm_backward_static: the partial sums of the gain/bias gradients, in a device
// array that exists from the moment the code object is loaded (one copy per GPU, held until the
// process ends), so that callers who cannot allocate device memory need no workspace.  In host code
// the name `scratch` is only a handle for hipGetSymbolAddress; kernels get the address it returns.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kWaves = 4;
constexpr int kBwdWaves = 8;  // LayerNorm backward: waves (= rows in flight) per workgroup

template <typename T, int NC>
__global__ __launch_bounds__(256) void ln_fwd_kernel(int rows, int h, const T* __restrict__ x,
                                                      const T* __restrict__ gain, const T* __restrict__ bias,
                                                      float eps, T* __restrict__ y, float* __restrict__ mean,
                                                      float* __restrict__ rstd, T* __restrict__ x_copy) {
  constexpr int V = Vec<T>::N;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * kWaves + wave;
  if (row >= rows) return;
  const T* xr = x + (size_t)row * h;
  // The row stays in registers as it is in memory (4 registers per 16-byte chunk; unpacked again for each of
  // the three passes): at 5120 bf16 columns that is 7 waves per SIMD instead of 2, and a wave lives for
  // little more than the latency of its loads, so the waves in flight are what the bandwidth comes from.
  u32x4 raw[NC];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < h) {
      raw[c] = Vec<T>::load_raw(xr + col);
      if (x_copy) Vec<T>::store_raw(x_copy + (size_t)row * h + col, raw[c]);
    }
  }

#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < h) {
      float v[V];
      Vec<T>::unpack(raw[c], v);
#pragma unroll
      for (int i = 0; i < V; ++i) sum += v[i];
    }
  }
  const float mu = wave_sum(sum) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < h) {
      float v[V];
      Vec<T>::unpack(raw[c], v);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const float d = v[i] - mu;
        sq += d * d;
      }
    }
  }
  const float rs = 1.0f / sqrtf(wave_sum(sq) / (float)h + eps);
  if (lane == 0) {
    mean[row] = mu;
    rstd[row] = rs;
  }
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < h) {
      float v[V], g[V], b[V], out[V];
      Vec<T>::unpack(raw[c], v);
      Vec<T>::load(gain + col, g);
      Vec<T>::load(bias + col, b);
#pragma unroll
      for (int i = 0; i < V; ++i) out[i] = g[i] * ((v[i] - mu) * rs) + b[i];
      Vec<T>::store(y + (size_t)row * h + col, out);
    }
  }
}

// dx = resid + rstd * (g - mean(g) - xhat * mean(g * xhat)),  g = dy * gain,  xhat = (x - mean) * rstd.
// A workgroup is 8 waves; WR of them share a row (wave w takes the column slice w % WR, NC chunks
// of 64 lanes x V elements), so a lane holds at most 3*V elements per tensor and 8/WR rows are in
// flight per workgroup.  The two row means are summed from the WR slices' wave sums in slice
// order through LDS.  Each lane keeps running column sums of dy * xhat and dy for its own
// columns; at the end the 8/WR waves that share a slice are folded in wave order and the
// workgroup writes one row of partials: partial[block][0..h) = d gain, [h..2h) = d bias.
template <typename T, int NC, int WR>
__global__ __launch_bounds__(kBwdWaves * 64) void ln_bwd_kernel(int rows, int h, const T* __restrict__ dy,
                                                      const T* x, const T* __restrict__ gain,
                                                      const float* __restrict__ mean, const float* __restrict__ rstd,
                                                      const T* resid, T* dx, float* __restrict__ partial) {
  constexpr int V = Vec<T>::N;
  constexpr int RG = kBwdWaves / WR;  // rows in flight
  extern __shared__ float red[];      // [2][WR * NC * V * 64], then the row sums [2][RG][WR][2]
  float (*stat)[RG][WR][2] = reinterpret_cast<float (*)[RG][WR][2]>(red + 2 * WR * NC * V * 64);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int rg = wave / WR, slice = wave % WR;
  const int col0 = (slice * NC * 64 + lane) * V;  // chunk c starts at col0 + c * 64 * V
  float pg[NC][V], pb[NC][V], gn[NC][V];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = col0 + c * 64 * V;
#pragma unroll
    for (int i = 0; i < V; ++i) pg[c][i] = pb[c][i] = gn[c][i] = 0.f;
    if (col < h) Vec<T>::load(gain + col, gn[c]);
  }
  int it = 0;
  for (int base = blockIdx.x * RG; base < rows; base += gridDim.x * RG, ++it) {
    const int row = base + rg;
    const bool live = row < rows;
    float xh[NC][V], g[NC][V], r[NC][V];
    float mu = 0.f, rs = 0.f, s1 = 0.f, s2 = 0.f;
    if (live) {
      mu = mean[row];
      rs = rstd[row];
      float xv[NC][V], d[NC][V];
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = col0 + c * 64 * V;
#pragma unroll
        for (int i = 0; i < V; ++i) xv[c][i] = d[c][i] = r[c][i] = 0.f;
        if (col < h) {
          Vec<T>::load(x + (size_t)row * h + col, xv[c]);
          Vec<T>::load(dy + (size_t)row * h + col, d[c]);
          if (resid) Vec<T>::load(resid + (size_t)row * h + col, r[c]);
        }
      }
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const bool in = col0 + c * 64 * V < h;  // lanes past the row end hold zeros, but mu != 0
#pragma unroll
        for (int i = 0; i < V; ++i) {
          xh[c][i] = in ? (xv[c][i] - mu) * rs : 0.f;
          g[c][i] = d[c][i] * gn[c][i];
          s1 += g[c][i];
          s2 += g[c][i] * xh[c][i];
          pg[c][i] += d[c][i] * xh[c][i];
          pb[c][i] += d[c][i];
        }
      }
      s1 = wave_sum(s1);
      s2 = wave_sum(s2);
    }
    if constexpr (WR > 1) {
      // Slots alternate with the iteration: a wave can only overwrite a slot two barriers after
      // every wave has read it.
      if (lane == 0) {
        stat[it & 1][rg][slice][0] = s1;
        stat[it & 1][rg][slice][1] = s2;
      }
      __syncthreads();
      s1 = s2 = 0.f;
#pragma unroll
      for (int w = 0; w < WR; ++w) {
        s1 += stat[it & 1][rg][w][0];
        s2 += stat[it & 1][rg][w][1];
      }
    }
    s1 /= (float)h;
    s2 /= (float)h;
    if (live) {
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = col0 + c * 64 * V;
        if (col < h) {
          float out[V];
#pragma unroll
          for (int i = 0; i < V; ++i) out[i] = r[c][i] + rs * (g[c][i] - s1 - xh[c][i] * s2);
          Vec<T>::store(dx + (size_t)row * h + col, out);
        }
      }
    }
  }
  // Fold: element (c, i) of lane l of slice s lives at red[((s*NC + c)*V + i) * 64 + (l + i*64/V) % 64]
  // (the d-bias half kHalf further on): a wave's 64 lanes hit 64 different words of one 64-word
  // line, and so does the write-out below, which walks i fastest.
  constexpr int kHalf = WR * NC * V * 64;
  for (int w = 0; w < RG; ++w) {
    if (rg == w) {
#pragma unroll
      for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const int a = ((slice * NC + c) * V + i) * 64 + ((lane + i * (64 / V)) & 63);
          if (w == 0) {
            red[a] = pg[c][i];
            red[kHalf + a] = pb[c][i];
          } else {
            red[a] += pg[c][i];
            red[kHalf + a] += pb[c][i];
          }
        }
      }
    }
    __syncthreads();
  }
  float* out = partial + (size_t)blockIdx.x * 2 * h;
  for (int j = threadIdx.x; j < h; j += kBwdWaves * 64) {
    const int i = j % V, l = (j / V) & 63, c = j / (V * 64);  // c counts chunks across slices
    const int a = (c * V + i) * 64 + ((l + i * (64 / V)) & 63);
    out[j] = red[a];
    out[h + j] = red[kHalf + a];
  }
}

// For every job j (blockIdx.y): out_a[i] += sum_p partial_j[p*stride + i] (i < split),
// out_b[i - split] += ... (i >= split).  A block handles 64 columns; its four waves each sum a
// contiguous quarter of the parts (loads are independent, so many are in flight), and the quarters
// are added in order 0,1,2,3: the summation order is fixed by (parts) alone.
__global__ __launch_bounds__(256) void sum_partials_kernel(LnPartialJobs jobs, int width, int split, size_t stride) {
  __shared__ float quarter[4][64];
  const int job = blockIdx.y;
  const float* __restrict__ partial = jobs.partial[job];
  const int parts = jobs.parts[job];
  const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + lane;
  const int per = (parts + 3) / 4, p0 = g * per, p1 = min(parts, p0 + per);
  float acc = 0.f;
  if (i < width) {
    int p = p0;
    for (; p + 8 <= p1; p += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(p + u) * stride + i];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; p < p1; ++p) acc += partial[(size_t)p * stride + i];
  }
  quarter[g][lane] = acc;
  __syncthreads();
  if (g == 0 && i < width) {
    const float total = ((quarter[0][lane] + quarter[1][lane]) + quarter[2][lane]) + quarter[3][lane];
    if (i < split) jobs.dgain[job][i] += total;
    else jobs.dbias[job][i - split] += total;
  }
}

// Column sums of up to four matrices with the same row count in one launch: out_j[c] += sum over
// rows of a_j[row][c].  A workgroup owns 64 columns of one matrix; its 256 threads form 256/LPR
// row slots of LPR lanes (16 bytes of a row each), slot s adds rows s, s + slots, ... in that
// order (sixteen loads in flight), and 64 threads then add the slots in slot order: the result
// depends on the shapes alone.
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(int rows, ColumnSumJobs jobs) {
  constexpr int V = Vec<T>::N, LPR = 64 / V, SLOTS = 256 / LPR, UNROLL = 16;
  __shared__ float red[SLOTS][64 + 1];
  int j = 0;
  while (j + 1 < jobs.count && (int)blockIdx.x >= jobs.first_block[j + 1]) ++j;
  const T* a = static_cast<const T*>(jobs.a[j]);
  const int n = jobs.n[j], lda = jobs.lda[j];
  const int slot = threadIdx.x / LPR, sub = (threadIdx.x % LPR) * V;
  const int col = ((int)blockIdx.x - jobs.first_block[j]) * 64 + sub;
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.f;
  if (col < n) {
    const T* p = a + col;
    int r = slot;
    for (; r + (UNROLL - 1) * SLOTS < rows; r += UNROLL * SLOTS) {
      float v[UNROLL][V];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) Vec<T>::load(p + (size_t)(r + u * SLOTS) * lda, v[u]);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += v[u][i];
    }
    for (; r < rows; r += SLOTS) {
      float v[V];
      Vec<T>::load(p + (size_t)r * lda, v);
#pragma unroll
      for (int i = 0; i < V; ++i) acc[i] += v[i];
    }
  }
#pragma unroll
  for (int i = 0; i < V; ++i) red[slot][sub + i] = acc[i];
  __syncthreads();
  const int c = ((int)blockIdx.x - jobs.first_block[j]) * 64 + threadIdx.x;
  if (threadIdx.x < 64 && c < n) {
    float total = 0.f;
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) total += red[sl][threadIdx.x];
    jobs.out[j][c] += total;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void copy_rows_kernel(int rows, int vec_cols, const T* __restrict__ src, int ld_src,
                                                         T* __restrict__ dst, int ld_dst) {
  constexpr int V = Vec<T>::N;
  const size_t total = (size_t)rows * vec_cols;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int r = (int)(i / vec_cols), c = (int)(i % vec_cols) * V;
    *reinterpret_cast<u32x4*>(dst + (size_t)r * ld_dst + c) = *reinterpret_cast<const u32x4*>(src + (size_t)r * ld_src + c);
  }
}

int pick_nc(int h, int vec) {
  const int need = (h + 64 * vec - 1) / (64 * vec);
  for (int nc : {1, 2, 3, 4, 6, 8, 12, 16, 20, 24})
    if (nc >= need) return nc;
  return 0;
}

// LayerNorm backward launch shape: WR waves per row so that a lane holds at most 3 chunks.
struct LnBwdShape {
  int nc, wr;
};
LnBwdShape ln_bwd_shape(int h, int vec) {
  const int need = (h + 64 * vec - 1) / (64 * vec);
  for (int wr : {1, 2, 4, 8}) {
    const int nc = (need + wr - 1) / wr;
    if (nc <= 3) return {nc, wr};
  }
  return {0, 0};
}

constexpr int kLnBwdMaxBlocks = 512;

int ln_bwd_blocks(int rows, int rows_in_flight) {
  const int b = (rows + rows_in_flight - 1) / rows_in_flight;
  return b < 1 ? 1 : (b > kLnBwdMaxBlocks ? kLnBwdMaxBlocks : b);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

#define PMC_LAUNCH_CHECK(what)                                                                \
  do {                                                                                        \
    hipError_t e_ = hipGetLastError();                                                        \
    if (e_ != hipSuccess) return fail(PMC_ERR_HIP, "%s launch failed: %s", what, hipGetErrorString(e_)); \
  } while (0)

template <typename T>
int ln_fwd_t(hipStream_t st, int rows, int h, const void* x, const void* gain, const void* bias, float eps, void* y,
             float* mean, float* rstd, void* x_copy) {
  const int nc = pick_nc(h, Vec<T>::N);
  dim3 grid((rows + kWaves - 1) / kWaves), block(256);
#define LN_FWD_CASE(NC)                                                                                          \
  case NC:                                                                                                       \
    ln_fwd_kernel<T, NC><<<grid, block, 0, st>>>(rows, h, (const T*)x, (const T*)gain, (const T*)bias, eps, (T*)y, \
                                                  mean, rstd, (T*)x_copy);                                       \
    break;
  switch (nc) {
    LN_FWD_CASE(1) LN_FWD_CASE(2) LN_FWD_CASE(3) LN_FWD_CASE(4) LN_FWD_CASE(6) LN_FWD_CASE(8) LN_FWD_CASE(12)
    LN_FWD_CASE(16) LN_FWD_CASE(20) LN_FWD_CASE(24)
    default:
      return fail(PMC_ERR_INVALID, "LayerNorm width %d too large", h);
  }
#undef LN_FWD_CASE
  PMC_LAUNCH_CHECK("layernorm_forward");
  return PMC_OK;
}

template <typename T>
int ln_bwd_t(hipStream_t st, int rows, int h, const void* dy, const void* x, const void* gain, const float* mean,
             const float* rstd, const void* resid, void* dx, float* dgain, float* dbias, float* partial,
             LnPartialJobs* defer) {
  const LnBwdShape sh = ln_bwd_shape(h, Vec<T>::N);
  if (!sh.nc) return fail(PMC_ERR_INVALID, "LayerNorm width %d too large", h);
  const int blocks = ln_bwd_blocks(rows, kBwdWaves / sh.wr);
  const size_t lds = ((size_t)2 * sh.wr * sh.nc * Vec<T>::N * 64 + 4 * kBwdWaves) * sizeof(float);
#define LN_BWD_CASE(NC, WR)                                                                                  \
  case NC * 16 + WR:                                                                                         \
    if (lds > 48 * 1024 &&                                                                                   \
        hipFuncSetAttribute(reinterpret_cast<const void*>(ln_bwd_kernel<T, NC, WR>),                         \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)             \
      return fail(PMC_ERR_HIP, "layernorm_backward: cannot reserve %zu bytes of LDS", lds);                  \
    ln_bwd_kernel<T, NC, WR><<<dim3(blocks), dim3(kBwdWaves * 64), lds, st>>>(                               \
        rows, h, (const T*)dy, (const T*)x, (const T*)gain, mean, rstd, (const T*)resid, (T*)dx, partial);   \
    break;
  switch (sh.nc * 16 + sh.wr) {
    LN_BWD_CASE(1, 1) LN_BWD_CASE(2, 1) LN_BWD_CASE(3, 1) LN_BWD_CASE(2, 2) LN_BWD_CASE(3, 2) LN_BWD_CASE(2, 4)
    LN_BWD_CASE(3, 4) LN_BWD_CASE(2, 8) LN_BWD_CASE(3, 8)
    default:
      return fail(PMC_ERR_INVALID, "LayerNorm width %d: no kernel for %d chunks x %d waves", h, sh.nc, sh.wr);
  }
#undef LN_BWD_CASE
  PMC_LAUNCH_CHECK("layernorm_backward");
  LnPartialJobs now;
  LnPartialJobs& jobs = defer ? *defer : now;
  if (jobs.count >= LnPartialJobs::kMax) return fail(PMC_ERR_INVALID, "layernorm_backward: too many deferred reductions");
  jobs.partial[jobs.count] = partial;
  jobs.dgain[jobs.count] = dgain;
  jobs.dbias[jobs.count] = dbias;
  jobs.parts[jobs.count] = blocks;
  ++jobs.count;
  return defer ? PMC_OK : layernorm_backward_reduce(st, h, jobs);
}

}  // namespace

int layernorm_forward(hipStream_t st, int dtype, int rows, int h, const void* x, const void* gain, const void* bias,
                      float eps, void* y, float* mean, float* rstd, void* x_copy) {
  if (rows <= 0 || h <= 0) return fail(PMC_ERR_INVALID, "layernorm: rows=%d h=%d", rows, h);
  const int vec = dtype == PMC_F32 ? 4 : 8;
  if (h % vec) return fail(PMC_ERR_INVALID, "layernorm: h=%d must be a multiple of %d", h, vec);
  if (!x || !gain || !bias || !y || !mean || !rstd) return fail(PMC_ERR_INVALID, "layernorm: NULL pointer");
  if (!aligned16(x) || !aligned16(gain) || !aligned16(bias) || !aligned16(y) || (x_copy && !aligned16(x_copy)))
    return fail(PMC_ERR_INVALID, "layernorm: pointers must be 16-byte aligned");
  if (dtype == PMC_F32) return ln_fwd_t<float>(st, rows, h, x, gain, bias, eps, y, mean, rstd, x_copy);
  if (dtype == PMC_BF16) return ln_fwd_t<bf16_t>(st, rows, h, x, gain, bias, eps, y, mean, rstd, x_copy);
  return fail(PMC_ERR_INVALID, "layernorm: bad dtype %d", dtype);
}

size_t layernorm_backward_scratch_floats(int rows, int h) {
  // Bound over both element types: at most one workgroup per row and kLnBwdMaxBlocks in all.
  return (size_t)ln_bwd_blocks(rows, 1) * 2 * h;
}

int layernorm_backward_reduce(hipStream_t st, int h, const LnPartialJobs& jobs) {
  if (jobs.count < 1 || jobs.count > LnPartialJobs::kMax) return fail(PMC_ERR_INVALID, "layernorm_backward_reduce: %d jobs", jobs.count);
  sum_partials_kernel<<<dim3((2 * h + 63) / 64, jobs.count), dim3(256), 0, st>>>(jobs, 2 * h, h, (size_t)2 * h);
  PMC_LAUNCH_CHECK("layernorm_backward reduce");
  return PMC_OK;
}

int layernorm_backward(hipStream_t st, int dtype, int rows, int h, const void* dy, const void* x, const void* gain,
                       const float* mean, const float* rstd, const void* resid, void* dx, float* dgain, float* dbias,
                       float* partial, LnPartialJobs* defer) {
  if (rows <= 0 || h <= 0) return fail(PMC_ERR_INVALID, "layernorm_backward: rows=%d h=%d", rows, h);
  const int vec = dtype == PMC_F32 ? 4 : 8;
  if (h % vec) return fail(PMC_ERR_INVALID, "layernorm_backward: h=%d must be a multiple of %d", h, vec);
  if (!dy || !x || !gain || !mean || !rstd || !dx || !dgain || !dbias || !partial)
    return fail(PMC_ERR_INVALID, "layernorm_backward: NULL pointer");
  if (!aligned16(dy) || !aligned16(x) || !aligned16(gain) || !aligned16(dx) || (resid && !aligned16(resid)))
    return fail(PMC_ERR_INVALID, "layernorm_backward: pointers must be 16-byte aligned");
  if (dtype == PMC_F32) return ln_bwd_t<float>(st, rows, h, dy, x, gain, mean, rstd, resid, dx, dgain, dbias, partial, defer);
  if (dtype == PMC_BF16) return ln_bwd_t<bf16_t>(st, rows, h, dy, x, gain, mean, rstd, resid, dx, dgain, dbias, partial, defer);
  return fail(PMC_ERR_INVALID, "layernorm_backward: bad dtype %d", dtype);
}

size_t layernorm_backward_static_scratch_bytes() { return kStaticScratchBytes; }

int layernorm_backward_static(hipStream_t st, int dtype, int rows, int h, const void* dy, const void* x, const void* gain,
                              const float* mean, const float* rstd, const void* resid, void* dx, float* dgain,
                              float* dbias) {
  if (rows <= 0 || h <= 0) return fail(PMC_ERR_INVALID, "layernorm_backward_static: rows=%d h=%d", rows, h);
  const size_t need = layernorm_backward_scratch_floats(rows, h) * sizeof(float);
  if (need > kStaticScratchBytes)
    return fail(PMC_ERR_NOMEM, "layernorm_backward_static: rows=%d x h=%d needs %zu bytes of scratch, the built-in array holds %zu",
                rows, h, need, kStaticScratchBytes);
  // The array has its own address on every GPU: looked up once per device, with that device current.
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static float* base[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(PMC_ERR_HIP, "layernorm_backward_static: cannot tell the current device");
  float* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!base[dev]) {
      void* p = nullptr;
      const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return fail(PMC_ERR_HIP, "layernorm_backward_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
      base[dev] = static_cast<float*>(p);
    }
    ptr = base[dev];
  }
  // every workgroup overwrites its whole row of partials before the reduction reads it: nothing
  // of the previous call's contents is read, nothing has to be cleared
  return layernorm_backward(st, dtype, rows, h, dy, x, gain, mean, rstd, resid, dx, dgain, dbias, ptr, nullptr);
}

int column_sums(hipStream_t st, int dtype, int rows, ColumnSumJobs jobs) {
  if (rows <= 0 || jobs.count < 1 || jobs.count > 4) return fail(PMC_ERR_INVALID, "column_sum: rows=%d jobs=%d", rows, jobs.count);
  if (dtype != PMC_F32 && dtype != PMC_BF16) return fail(PMC_ERR_INVALID, "column_sum: bad dtype %d", dtype);
  const int vec = dtype == PMC_F32 ? 4 : 8;
  int blocks = 0;
  for (int j = 0; j < jobs.count; ++j) {
    const int n = jobs.n[j], lda = jobs.lda[j];
    if (n <= 0 || n % vec || lda % vec || lda < n)
      return fail(PMC_ERR_INVALID, "column_sum: n=%d lda=%d must be multiples of %d", n, lda, vec);
    if (!jobs.a[j] || !jobs.out[j] || !aligned16(jobs.a[j])) return fail(PMC_ERR_INVALID, "column_sum: bad pointer");
    jobs.first_block[j] = blocks;
    blocks += (n + 63) / 64;
  }
  for (int j = jobs.count; j < 5; ++j) jobs.first_block[j] = blocks;
  if (dtype == PMC_F32) colsum_kernel<float><<<dim3(blocks), dim3(256), 0, st>>>(rows, jobs);
  else colsum_kernel<bf16_t><<<dim3(blocks), dim3(256), 0, st>>>(rows, jobs);
  PMC_LAUNCH_CHECK("column_sum");
  return PMC_OK;
}

int column_sum(hipStream_t st, int dtype, int rows, int n, const void* a, int lda, float* out) {
  ColumnSumJobs jobs = {};
  jobs.count = 1;
  jobs.a[0] = a;
  jobs.out[0] = out;
  jobs.n[0] = n;
  jobs.lda[0] = lda;
  return column_sums(st, dtype, rows, jobs);
}

int copy_rows(hipStream_t st, int dtype, int rows, int cols, const void* src, int ld_src, void* dst, int ld_dst) {
  const int vec = dtype == PMC_F32 ? 4 : 8;
  if (rows <= 0 || cols <= 0 || cols % vec || ld_src % vec || ld_dst % vec)
    return fail(PMC_ERR_INVALID, "copy_rows: bad shape rows=%d cols=%d", rows, cols);
  if (!aligned16(src) || !aligned16(dst)) return fail(PMC_ERR_INVALID, "copy_rows: pointers must be 16-byte aligned");
  const size_t total = (size_t)rows * (cols / vec);
  int blocks = (int)((total + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  if (dtype == PMC_F32) copy_rows_kernel<float><<<dim3(blocks), dim3(256), 0, st>>>(rows, cols / vec, (const float*)src, ld_src, (float*)dst, ld_dst);
  else copy_rows_kernel<bf16_t><<<dim3(blocks), dim3(256), 0, st>>>(rows, cols / vec, (const bf16_t*)src, ld_src, (bf16_t*)dst, ld_dst);
  PMC_LAUNCH_CHECK("copy_rows");
  return PMC_OK;
}

}  // namespace k
}  // namespace pmc
