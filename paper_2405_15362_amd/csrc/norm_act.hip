// Row-wise kernels bounded by HBM bandwidth: LayerNorm forward, LayerNorm input-gradient (with the
// gain/bias gradient partial sums), column sums for the bias gradients, and a pitched row copy.
// One 64-lane wave owns a row; all reductions along a row are wave shuffles.  Reductions across
// rows go through fixed-order partial sums, so results do not depend on scheduling.
#include "dev_common.h"
#include "kernels.h"

namespace pmc {
namespace k {
namespace {

constexpr int kWaves = 4;

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
  float v[NC][V];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < h) {
      Vec<T>::load(xr + col, v[c]);
      if (x_copy) Vec<T>::store(x_copy + (size_t)row * h + col, v[c]);
#pragma unroll
      for (int i = 0; i < V; ++i) sum += v[c][i];
    }
  }
  const float mu = wave_sum(sum) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < h) {
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const float d = v[c][i] - mu;
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
      float g[V], b[V], out[V];
      Vec<T>::load(gain + col, g);
      Vec<T>::load(bias + col, b);
#pragma unroll
      for (int i = 0; i < V; ++i) out[i] = g[i] * ((v[c][i] - mu) * rs) + b[i];
      Vec<T>::store(y + (size_t)row * h + col, out);
    }
  }
}

// dx = resid + rstd * (g - mean(g) - xhat * mean(g * xhat)),  g = dy * gain,  xhat = (x - mean) * rstd.
// Each wave walks rows blockIdx*4+wave, +4*gridDim, ... and keeps, per lane, the running column
// sums of dy * xhat and dy for its own columns; the block then folds its four waves in wave
// order and writes one row of partials: partial[block][0..h) = d gain, [h..2h) = d bias.
template <typename T, int NC>
__global__ __launch_bounds__(256) void ln_bwd_kernel(int rows, int h, const T* __restrict__ dy,
                                                      const T* x, const T* __restrict__ gain,
                                                      const float* __restrict__ mean, const float* __restrict__ rstd,
                                                      const T* resid, T* dx, float* __restrict__ partial) {
  constexpr int V = Vec<T>::N;
  extern __shared__ float red[];  // [2][h]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float pg[NC][V], pb[NC][V], gn[NC][V];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int col = (c * 64 + lane) * V;
#pragma unroll
    for (int i = 0; i < V; ++i) pg[c][i] = pb[c][i] = gn[c][i] = 0.f;
    if (col < h) Vec<T>::load(gain + col, gn[c]);
  }
  for (int row = blockIdx.x * kWaves + wave; row < rows; row += gridDim.x * kWaves) {
    const float mu = mean[row], rs = rstd[row];
    float xh[NC][V], g[NC][V];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int col = (c * 64 + lane) * V;
      if (col < h) {
        float xv[V], d[V];
        Vec<T>::load(x + (size_t)row * h + col, xv);
        Vec<T>::load(dy + (size_t)row * h + col, d);
#pragma unroll
        for (int i = 0; i < V; ++i) {
          xh[c][i] = (xv[i] - mu) * rs;
          g[c][i] = d[i] * gn[c][i];
          s1 += g[c][i];
          s2 += g[c][i] * xh[c][i];
          pg[c][i] += d[i] * xh[c][i];
          pb[c][i] += d[i];
        }
      }
    }
    s1 = wave_sum(s1) / (float)h;
    s2 = wave_sum(s2) / (float)h;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int col = (c * 64 + lane) * V;
      if (col < h) {
        float r[V], out[V];
        if (resid) {
          Vec<T>::load(resid + (size_t)row * h + col, r);
        } else {
#pragma unroll
          for (int i = 0; i < V; ++i) r[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < V; ++i) out[i] = r[i] + rs * (g[c][i] - s1 - xh[c][i] * s2);
        Vec<T>::store(dx + (size_t)row * h + col, out);
      }
    }
  }
  for (int w = 0; w < kWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int col = (c * 64 + lane) * V;
        if (col < h) {
#pragma unroll
          for (int i = 0; i < V; ++i) {
            if (w == 0) {
              red[col + i] = pg[c][i];
              red[h + col + i] = pb[c][i];
            } else {
              red[col + i] += pg[c][i];
              red[h + col + i] += pb[c][i];
            }
          }
        }
      }
    }
    __syncthreads();
  }
  float* out = partial + (size_t)blockIdx.x * 2 * h;
  for (int i = threadIdx.x; i < 2 * h; i += 256) out[i] = red[i];
}

// out_a[i] += sum_p partial[p*stride + i] (i < split), out_b[i - split] += ... (i >= split).
// A block handles 64 columns; its four waves each sum a contiguous quarter of the parts (loads
// are independent, so many are in flight), and the quarters are added in order 0,1,2,3: the
// summation order is fixed by (parts) alone.
__global__ __launch_bounds__(256) void sum_partials_kernel(int parts, int width, int split, size_t stride,
                                                            const float* __restrict__ partial,
                                                            float* __restrict__ out_a, float* __restrict__ out_b) {
  __shared__ float quarter[4][64];
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
    if (i < split) out_a[i] += total;
    else out_b[i - split] += total;
  }
}

// partial[blockIdx.y][col] = sum over the block's slice of rows of a[row][col].
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(int rows, int n, const T* __restrict__ a, int lda,
                                                      int rows_per_part, float* __restrict__ partial) {
  constexpr int V = Vec<T>::N;
  const int col = (blockIdx.x * 256 + threadIdx.x) * V;
  if (col >= n) return;
  const int r0 = blockIdx.y * rows_per_part;
  const int r1 = min(rows, r0 + rows_per_part);
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.f;
  for (int r = r0; r < r1; ++r) {
    float v[V];
    Vec<T>::load(a + (size_t)r * lda + col, v);
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] += v[i];
  }
#pragma unroll
  for (int i = 0; i < V; ++i) partial[(size_t)blockIdx.y * n + col + i] = acc[i];
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
  for (int nc : {1, 2, 3, 4, 6, 8, 12, 16})
    if (nc >= need) return nc;
  return 0;
}

int ln_bwd_blocks(int rows) {
  int b = (rows + 2 * kWaves - 1) / (2 * kWaves);
  return b < 1 ? 1 : (b > 256 ? 256 : b);
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
    LN_FWD_CASE(16)
    default:
      return fail(PMC_ERR_INVALID, "LayerNorm width %d too large", h);
  }
#undef LN_FWD_CASE
  PMC_LAUNCH_CHECK("layernorm_forward");
  return PMC_OK;
}

template <typename T>
int ln_bwd_t(hipStream_t st, int rows, int h, const void* dy, const void* x, const void* gain, const float* mean,
             const float* rstd, const void* resid, void* dx, float* dgain, float* dbias, float* partial) {
  const int nc = pick_nc(h, Vec<T>::N);
  const int blocks = ln_bwd_blocks(rows);
  const size_t lds = (size_t)2 * h * sizeof(float);
#define LN_BWD_CASE(NC)                                                                                       \
  case NC:                                                                                                    \
    ln_bwd_kernel<T, NC><<<dim3(blocks), dim3(256), lds, st>>>(rows, h, (const T*)dy, (const T*)x, (const T*)gain, \
                                                               mean, rstd, (const T*)resid, (T*)dx, partial); \
    break;
  switch (nc) {
    LN_BWD_CASE(1) LN_BWD_CASE(2) LN_BWD_CASE(3) LN_BWD_CASE(4) LN_BWD_CASE(6) LN_BWD_CASE(8) LN_BWD_CASE(12)
    LN_BWD_CASE(16)
    default:
      return fail(PMC_ERR_INVALID, "LayerNorm width %d too large", h);
  }
#undef LN_BWD_CASE
  PMC_LAUNCH_CHECK("layernorm_backward");
  sum_partials_kernel<<<dim3((2 * h + 63) / 64), dim3(256), 0, st>>>(blocks, 2 * h, h, (size_t)2 * h, partial, dgain,
                                                                       dbias);
  PMC_LAUNCH_CHECK("layernorm_backward reduce");
  return PMC_OK;
}

int colsum_parts(int rows) {
  int p = rows / 16;
  return p < 1 ? 1 : (p > 128 ? 128 : p);
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

size_t layernorm_backward_scratch_floats(int rows, int h) { return (size_t)ln_bwd_blocks(rows) * 2 * h; }

int layernorm_backward(hipStream_t st, int dtype, int rows, int h, const void* dy, const void* x, const void* gain,
                       const float* mean, const float* rstd, const void* resid, void* dx, float* dgain, float* dbias,
                       float* partial) {
  if (rows <= 0 || h <= 0) return fail(PMC_ERR_INVALID, "layernorm_backward: rows=%d h=%d", rows, h);
  const int vec = dtype == PMC_F32 ? 4 : 8;
  if (h % vec) return fail(PMC_ERR_INVALID, "layernorm_backward: h=%d must be a multiple of %d", h, vec);
  if (!dy || !x || !gain || !mean || !rstd || !dx || !dgain || !dbias || !partial)
    return fail(PMC_ERR_INVALID, "layernorm_backward: NULL pointer");
  if (!aligned16(dy) || !aligned16(x) || !aligned16(gain) || !aligned16(dx) || (resid && !aligned16(resid)))
    return fail(PMC_ERR_INVALID, "layernorm_backward: pointers must be 16-byte aligned");
  if ((size_t)2 * h * sizeof(float) > 64 * 1024) return fail(PMC_ERR_INVALID, "layernorm_backward: h=%d too large", h);
  if (dtype == PMC_F32) return ln_bwd_t<float>(st, rows, h, dy, x, gain, mean, rstd, resid, dx, dgain, dbias, partial);
  if (dtype == PMC_BF16) return ln_bwd_t<bf16_t>(st, rows, h, dy, x, gain, mean, rstd, resid, dx, dgain, dbias, partial);
  return fail(PMC_ERR_INVALID, "layernorm_backward: bad dtype %d", dtype);
}

size_t column_sum_scratch_floats(int rows, int n) { return (size_t)colsum_parts(rows) * n; }

int column_sum(hipStream_t st, int dtype, int rows, int n, const void* a, int lda, float* out, float* partial) {
  if (rows <= 0 || n <= 0) return fail(PMC_ERR_INVALID, "column_sum: rows=%d n=%d", rows, n);
  const int vec = dtype == PMC_F32 ? 4 : 8;
  if (n % vec || lda % vec || lda < n) return fail(PMC_ERR_INVALID, "column_sum: n=%d lda=%d must be multiples of %d", n, lda, vec);
  if (!a || !out || !partial || !aligned16(a)) return fail(PMC_ERR_INVALID, "column_sum: bad pointer");
  const int parts = colsum_parts(rows);
  const int rpp = (rows + parts - 1) / parts;
  dim3 grid((n / vec + 255) / 256, parts), block(256);
  if (dtype == PMC_F32) colsum_kernel<float><<<grid, block, 0, st>>>(rows, n, (const float*)a, lda, rpp, partial);
  else if (dtype == PMC_BF16) colsum_kernel<bf16_t><<<grid, block, 0, st>>>(rows, n, (const bf16_t*)a, lda, rpp, partial);
  else return fail(PMC_ERR_INVALID, "column_sum: bad dtype %d", dtype);
  PMC_LAUNCH_CHECK("column_sum");
  sum_partials_kernel<<<dim3((n + 63) / 64), dim3(256), 0, st>>>(parts, n, n, (size_t)n, partial, out, out);
  PMC_LAUNCH_CHECK("column_sum reduce");
  return PMC_OK;
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
