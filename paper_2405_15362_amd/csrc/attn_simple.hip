// Flash-style attention in plain fp32 arithmetic (no matrix cores), streaming over key tiles with
// an online softmax so that no s x s matrix is ever stored.  This is the PMC_F32-mode path, where
// results must agree with the fp64 oracle to 1e-5.  Packed qkv is [batch*seq, 3h], h = heads*dh.
//
// Backward is two kernels so that every output element has exactly one writer and a fixed
// summation order: dq per query tile (also emits delta = rowsum(dO * O)), then dk/dv per key tile,
// written in place over k and v (a key tile is read only by the workgroup that owns it).
#include "dev_common.h"
#include "kernels.h"

namespace pmc {
namespace k {
namespace {

constexpr int kMaxDh = 128;
constexpr int kPitch = kMaxDh + 1;
constexpr int TQ = 16;   // rows owned by a workgroup
constexpr int TK = 32;   // streamed tile

template <typename T>
__device__ __forceinline__ void load_tile(float (*dst)[kPitch], const T* base, size_t pitch, int row0, int nrows,
                                          int row_limit, int dh) {
  for (int i = threadIdx.x; i < nrows * dh; i += 256) {
    const int r = i / dh, c = i % dh;
    const int gr = row0 + r;
    dst[r][c] = gr < row_limit ? to_f32(base[(size_t)gr * pitch + c]) : 0.f;
  }
}

__device__ __forceinline__ float group16_sum(float v) {
  v += __shfl_xor(v, 8, 64); v += __shfl_xor(v, 4, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 1, 64);
  return v;
}
__device__ __forceinline__ float group16_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 8, 64)); v = fmaxf(v, __shfl_xor(v, 4, 64));
  v = fmaxf(v, __shfl_xor(v, 2, 64)); v = fmaxf(v, __shfl_xor(v, 1, 64));
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simple(int seq, int heads, int dh, int causal, const T* __restrict__ qkv,
                                                        T* __restrict__ o, float* __restrict__ lse) {
  __shared__ float qs[TQ][kPitch], ks[TK][kPitch], vs[TK][kPitch], ps[TQ][TK + 1];
  const int h = heads * dh, q0 = blockIdx.x * TQ, head = blockIdx.y, b = blockIdx.z;
  const size_t pitch = (size_t)3 * h;
  const T* base = qkv + (size_t)b * seq * pitch + (size_t)head * dh;
  const int i = threadIdx.x / 16, j = threadIdx.x % 16;
  const int qi = q0 + i;
  const float sigma = 1.0f / sqrtf((float)dh);
  load_tile(qs, base, pitch, q0, TQ, seq, dh);
  float m = -INFINITY, l = 0.f, acc[kMaxDh / 16];
#pragma unroll
  for (int c = 0; c < kMaxDh / 16; ++c) acc[c] = 0.f;
  const int kend = causal ? min(seq, q0 + TQ) : seq;
  for (int k0 = 0; k0 < kend; k0 += TK) {
    __syncthreads();
    load_tile(ks, base + h, pitch, k0, TK, seq, dh);
    load_tile(vs, base + 2 * h, pitch, k0, TK, seq, dh);
    __syncthreads();
    float s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int jj = j + 16 * t, kj = k0 + jj;
      float d = 0.f;
      for (int c = 0; c < dh; ++c) d = fmaf(qs[i][c], ks[jj][c], d);
      s[t] = (kj < seq && (!causal || kj <= qi)) ? d * sigma : -INFINITY;
    }
    const float tile_max = group16_max(fmaxf(s[0], s[1]));
    const float m_new = fmaxf(m, tile_max);
    // m_new is finite whenever this row has seen an unmasked key; rows past the end of the
    // sequence stay at -inf and are never written.
    const float scale = (m_new == -INFINITY) ? 1.f : expf(m - m_new);
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const float p = (s[t] == -INFINITY) ? 0.f : expf(s[t] - m_new);
      ps[i][j + 16 * t] = p;
      psum += p;
    }
    l = l * scale + group16_sum(psum);
    m = m_new;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kMaxDh / 16; ++c) {
      const int col = j + 16 * c;
      if (col < dh) {
        float a = acc[c] * scale;
        for (int jj = 0; jj < TK; ++jj) a = fmaf(ps[i][jj], vs[jj][col], a);
        acc[c] = a;
      }
    }
  }
  if (qi < seq) {
    const float inv = 1.0f / l;
#pragma unroll
    for (int c = 0; c < kMaxDh / 16; ++c) {
      const int col = j + 16 * c;
      if (col < dh) o[((size_t)b * seq + qi) * h + (size_t)head * dh + col] = from_f32<T>(acc[c] * inv);
    }
    if (j == 0) lse[((size_t)b * heads + head) * seq + qi] = m + logf(l);
  }
}

// dq[i] = sigma * sum_j dS[i][j] k[j],  dS = P * (dP - delta),  P = exp(S - lse),  dP = dO . V^T.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple(int seq, int heads, int dh, int causal,
                                                           const T* __restrict__ qkv, const T* __restrict__ o,
                                                           const float* __restrict__ lse, const T* __restrict__ d_o,
                                                           T* __restrict__ dq, float* __restrict__ delta) {
  __shared__ float qs[TQ][kPitch], dos[TQ][kPitch], ks[TK][kPitch], vs[TK][kPitch], ps[TQ][TK + 1];
  const int h = heads * dh, q0 = blockIdx.x * TQ, head = blockIdx.y, b = blockIdx.z;
  const size_t pitch = (size_t)3 * h;
  const T* base = qkv + (size_t)b * seq * pitch + (size_t)head * dh;
  const T* dob = d_o + (size_t)b * seq * h + (size_t)head * dh;
  const T* ob = o + (size_t)b * seq * h + (size_t)head * dh;
  const int i = threadIdx.x / 16, j = threadIdx.x % 16;
  const int qi = q0 + i;
  const float sigma = 1.0f / sqrtf((float)dh);
  load_tile(qs, base, pitch, q0, TQ, seq, dh);
  load_tile(dos, dob, (size_t)h, q0, TQ, seq, dh);
  __syncthreads();
  float dl = 0.f;
  if (qi < seq)
    for (int c = j; c < dh; c += 16) dl = fmaf(dos[i][c], to_f32(ob[(size_t)qi * h + c]), dl);
  dl = group16_sum(dl);
  const float my_lse = qi < seq ? lse[((size_t)b * heads + head) * seq + qi] : 0.f;
  if (j == 0 && qi < seq) delta[((size_t)b * heads + head) * seq + qi] = dl;
  float acc[kMaxDh / 16];
#pragma unroll
  for (int c = 0; c < kMaxDh / 16; ++c) acc[c] = 0.f;
  const int kend = causal ? min(seq, q0 + TQ) : seq;
  for (int k0 = 0; k0 < kend; k0 += TK) {
    __syncthreads();
    load_tile(ks, base + h, pitch, k0, TK, seq, dh);
    load_tile(vs, base + 2 * h, pitch, k0, TK, seq, dh);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int jj = j + 16 * t, kj = k0 + jj;
      float d = 0.f, dp = 0.f;
      for (int c = 0; c < dh; ++c) {
        d = fmaf(qs[i][c], ks[jj][c], d);
        dp = fmaf(dos[i][c], vs[jj][c], dp);
      }
      const bool live = qi < seq && kj < seq && (!causal || kj <= qi);
      const float p = live ? expf(d * sigma - my_lse) : 0.f;
      ps[i][jj] = p * (dp - dl);
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kMaxDh / 16; ++c) {
      const int col = j + 16 * c;
      if (col < dh) {
        float a = acc[c];
        for (int jj = 0; jj < TK; ++jj) a = fmaf(ps[i][jj], ks[jj][col], a);
        acc[c] = a;
      }
    }
  }
  if (qi < seq) {
#pragma unroll
    for (int c = 0; c < kMaxDh / 16; ++c) {
      const int col = j + 16 * c;
      if (col < dh) dq[((size_t)b * seq + qi) * h + (size_t)head * dh + col] = from_f32<T>(acc[c] * sigma);
    }
  }
}

// For a tile of 16 keys: dv[j] = sum_i P[i][j] dO[i],  dk[j] = sigma * sum_i dS[i][j] q[i];
// written over v[j] and k[j] inside the packed buffer.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple(int seq, int heads, int dh, int causal, const T* qkv,
                                                            const float* __restrict__ lse,
                                                            const float* __restrict__ delta,
                                                            const T* __restrict__ d_o, T* dqkv) {
  __shared__ float ks[TQ][kPitch], vs[TQ][kPitch], qs[TK][kPitch], dos[TK][kPitch], pT[TQ][TK + 1], dsT[TQ][TK + 1];
  __shared__ float lse_s[TK], delta_s[TK];
  const int h = heads * dh, k0 = blockIdx.x * TQ, head = blockIdx.y, b = blockIdx.z;
  const size_t pitch = (size_t)3 * h;
  const T* base = qkv + (size_t)b * seq * pitch + (size_t)head * dh;
  const T* dob = d_o + (size_t)b * seq * h + (size_t)head * dh;
  const int jk = threadIdx.x / 16, jq = threadIdx.x % 16;
  const int kj = k0 + jk;
  const float sigma = 1.0f / sqrtf((float)dh);
  load_tile(ks, base + h, pitch, k0, TQ, seq, dh);
  load_tile(vs, base + 2 * h, pitch, k0, TQ, seq, dh);
  float accv[kMaxDh / 16], acck[kMaxDh / 16];
#pragma unroll
  for (int c = 0; c < kMaxDh / 16; ++c) accv[c] = acck[c] = 0.f;
  const int qstart = causal ? (k0 / TK) * TK : 0;
  for (int q0 = qstart; q0 < seq; q0 += TK) {
    __syncthreads();
    load_tile(qs, base, pitch, q0, TK, seq, dh);
    load_tile(dos, dob, (size_t)h, q0, TK, seq, dh);
    if (threadIdx.x < TK) {
      const int qi = q0 + threadIdx.x;
      lse_s[threadIdx.x] = qi < seq ? lse[((size_t)b * heads + head) * seq + qi] : 0.f;
      delta_s[threadIdx.x] = qi < seq ? delta[((size_t)b * heads + head) * seq + qi] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int ii = jq + 16 * t, qi = q0 + ii;
      float d = 0.f, dp = 0.f;
      for (int c = 0; c < dh; ++c) {
        d = fmaf(qs[ii][c], ks[jk][c], d);
        dp = fmaf(dos[ii][c], vs[jk][c], dp);
      }
      const bool live = qi < seq && kj < seq && (!causal || kj <= qi);
      const float p = live ? expf(d * sigma - lse_s[ii]) : 0.f;
      pT[jk][ii] = p;
      dsT[jk][ii] = p * (dp - delta_s[ii]);
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kMaxDh / 16; ++c) {
      const int col = jq + 16 * c;
      if (col < dh) {
        float av = accv[c], ak = acck[c];
        for (int ii = 0; ii < TK; ++ii) {
          av = fmaf(pT[jk][ii], dos[ii][col], av);
          ak = fmaf(dsT[jk][ii], qs[ii][col], ak);
        }
        accv[c] = av;
        acck[c] = ak;
      }
    }
  }
  if (kj < seq) {
    T* out = dqkv + ((size_t)b * seq + kj) * pitch + (size_t)head * dh;
#pragma unroll
    for (int c = 0; c < kMaxDh / 16; ++c) {
      const int col = jq + 16 * c;
      if (col < dh) {
        out[h + col] = from_f32<T>(acck[c] * sigma);
        out[2 * h + col] = from_f32<T>(accv[c]);
      }
    }
  }
}

int check(const char* what, int batch, int seq, int heads, int dh) {
  if (batch <= 0 || seq <= 0 || heads <= 0) return fail(PMC_ERR_INVALID, "%s: batch=%d seq=%d heads=%d", what, batch, seq, heads);
  if (dh <= 0 || dh > kMaxDh) return fail(PMC_ERR_INVALID, "%s: head size %d not in 1..%d", what, dh, kMaxDh);
  if (heads > 65535 || batch > 65535) return fail(PMC_ERR_INVALID, "%s: heads/batch exceed the grid limit", what);
  return PMC_OK;
}

}  // namespace

int attention_forward_simple(hipStream_t st, int dtype, int batch, int seq, int heads, int dh, int causal,
                             const void* qkv, void* o, float* lse) {
  if (int rc = check("attention_forward", batch, seq, heads, dh)) return rc;
  dim3 grid((seq + TQ - 1) / TQ, heads, batch), block(256);
  if (dtype == PMC_F32) attn_fwd_simple<float><<<grid, block, 0, st>>>(seq, heads, dh, causal, (const float*)qkv, (float*)o, lse);
  else attn_fwd_simple<bf16_t><<<grid, block, 0, st>>>(seq, heads, dh, causal, (const bf16_t*)qkv, (bf16_t*)o, lse);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "attention_forward launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

// dq_stage: [batch*seq, h] storage type; delta: fp32 [batch, heads, seq].
int attention_backward_simple(hipStream_t st, int dtype, int batch, int seq, int heads, int dh, int causal,
                              const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                              void* dq_stage, float* delta) {
  if (int rc = check("attention_backward", batch, seq, heads, dh)) return rc;
  dim3 grid((seq + TQ - 1) / TQ, heads, batch), block(256);
  if (dtype == PMC_F32) {
    attn_bwd_dq_simple<float><<<grid, block, 0, st>>>(seq, heads, dh, causal, (const float*)qkv, (const float*)o, lse,
                                                      (const float*)d_o, (float*)dq_stage, delta);
    attn_bwd_dkv_simple<float><<<grid, block, 0, st>>>(seq, heads, dh, causal, (const float*)qkv, lse, delta,
                                                       (const float*)d_o, (float*)dqkv);
  } else {
    attn_bwd_dq_simple<bf16_t><<<grid, block, 0, st>>>(seq, heads, dh, causal, (const bf16_t*)qkv, (const bf16_t*)o, lse,
                                                       (const bf16_t*)d_o, (bf16_t*)dq_stage, delta);
    attn_bwd_dkv_simple<bf16_t><<<grid, block, 0, st>>>(seq, heads, dh, causal, (const bf16_t*)qkv, lse, delta,
                                                        (const bf16_t*)d_o, (bf16_t*)dqkv);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "attention_backward launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

}  // namespace k
}  // namespace pmc
