// fp32 reference-mode GEMM (plain FMA, LDS-tiled).  Used only in PMC_F32 mode, where results must
// agree with the fp64 oracle to 1e-5, which rules out the bf16 matrix cores.  Any sizes.
#include "dev_common.h"
#include "kernels.h"

namespace pmc {
namespace k {
namespace {

constexpr int BM = 64, BN = 64, BK = 16;

// C[M,N] (+)= op(A) . op(B); TA: A stored [K,M]; TB: B stored [N,K].  Sum over k in ascending order.
template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(int M, int N, int K, const float* __restrict__ A, int lda,
                                                        const float* __restrict__ B, int ldb, float* C, int ldc,
                                                        int epi, const float* __restrict__ bias, const float* resid,
                                                        float* aux) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = tid; i < BM * BK; i += 256) {
      int m, k;
      if (TA) { m = i % BM; k = i / BM; } else { k = i % BK; m = i / BK; }
      const int gm = m0 + m, gk = k0 + k;
      float v = 0.f;
      if (gm < M && gk < K) v = TA ? A[(size_t)gk * lda + gm] : A[(size_t)gm * lda + gk];
      As[k][m] = v;
    }
    for (int i = tid; i < BN * BK; i += 256) {
      int n, k;
      if (TB) { k = i % BK; n = i / BK; } else { n = i % BN; k = i / BN; }
      const int gn = n0 + n, gk = k0 + k;
      float v = 0.f;
      if (gn < N && gk < K) v = TB ? B[(size_t)gn * ldb + gk] : B[(size_t)gk * ldb + gn];
      Bs[k][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      const size_t idx = (size_t)gm * ldc + gn;
      float v = acc[i][j];
      switch (epi) {
        case PMC_EPI_NONE: C[idx] = v; break;
        case PMC_EPI_BIAS: C[idx] = v + bias[gn]; break;
        case PMC_EPI_BIAS_RESID: C[idx] = v + bias[gn] + resid[idx]; break;
        case PMC_EPI_BIAS_GELU: v += bias[gn]; C[idx] = v; aux[idx] = gelu_f(v); break;
        case PMC_EPI_DGELU: C[idx] = v * gelu_grad_f(aux[idx]); break;
        case PMC_EPI_ACCUM_F32: C[idx] += v; break;
        case PMC_EPI_BIAS_GELU_GRAD: v += bias[gn]; C[idx] = gelu_grad_f(v); aux[idx] = gelu_f(v); break;
        case PMC_EPI_MUL: C[idx] = v * aux[idx]; break;
      }
    }
  }
}

}  // namespace

int gemm_f32(hipStream_t st, const GemmArgs& a) {
  dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM), block(256);
  const float* A = (const float*)a.A;
  const float* B = (const float*)a.B;
  float* C = (float*)a.C;
  const float* bias = (const float*)a.bias;
  const float* resid = (const float*)a.resid;
  float* aux = (float*)a.aux;
#define GO(TA, TB) \
  gemm_f32_kernel<TA, TB><<<grid, block, 0, st>>>(a.M, a.N, a.K, A, a.lda, B, a.ldb, C, a.ldc, a.epilogue, bias, resid, aux)
  if (!a.trans_a && !a.trans_b) GO(false, false);
  else if (!a.trans_a && a.trans_b) GO(false, true);
  else if (a.trans_a && !a.trans_b) GO(true, false);
  else GO(true, true);
#undef GO
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "gemm_f32 launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

// Shape and pointer checks common to both precisions, then dispatch.
int gemm(hipStream_t st, const GemmArgs& a) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(PMC_ERR_INVALID, "gemm: M=%d N=%d K=%d", a.M, a.N, a.K);
  if (!a.A || !a.B || !a.C) return fail(PMC_ERR_INVALID, "gemm: NULL operand");
  const int a_cols = a.trans_a ? a.M : a.K, b_cols = a.trans_b ? a.K : a.N;
  if (a.lda < a_cols || a.ldb < b_cols || a.ldc < a.N)
    return fail(PMC_ERR_INVALID, "gemm: pitch too small (lda=%d ldb=%d ldc=%d)", a.lda, a.ldb, a.ldc);
  switch (a.epilogue) {
    case PMC_EPI_NONE:
    case PMC_EPI_ACCUM_F32:
      break;
    case PMC_EPI_BIAS:
      if (!a.bias) return fail(PMC_ERR_INVALID, "gemm: bias epilogue without bias");
      break;
    case PMC_EPI_BIAS_RESID:
      if (!a.bias || !a.resid) return fail(PMC_ERR_INVALID, "gemm: bias+residual epilogue needs both");
      break;
    case PMC_EPI_BIAS_GELU:
    case PMC_EPI_BIAS_GELU_GRAD:
      if (!a.bias || !a.aux) return fail(PMC_ERR_INVALID, "gemm: bias+gelu epilogue needs bias and aux");
      break;
    case PMC_EPI_DGELU:
    case PMC_EPI_MUL:
      if (!a.aux) return fail(PMC_ERR_INVALID, "gemm: this epilogue needs aux");
      break;
    default:
      return fail(PMC_ERR_INVALID, "gemm: unknown epilogue %d", a.epilogue);
  }
  if (a.dtype == PMC_F32) return gemm_f32(st, a);
  if (a.dtype == PMC_BF16) return gemm_bf16(st, a);
  return fail(PMC_ERR_INVALID, "gemm: bad dtype %d", a.dtype);
}

}  // namespace k
}  // namespace pmc
