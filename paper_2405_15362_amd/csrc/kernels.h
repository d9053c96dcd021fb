// Host-callable launchers of the HIP kernels.  Every launcher validates what its kernel assumes
// about shapes and alignment, enqueues on `stream` and returns a pmc_status.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

#include "pmc_internal.h"

namespace pmc {
namespace k {

// One-time reservation of a kernel's dynamic LDS, reachable from several host threads at once: the
// flag is atomic and the attribute call is idempotent, so a race at first use only repeats the call.
template <typename Kern>
int reserve_lds(Kern kern, size_t bytes, std::atomic<bool>& done, const char* what) {
  if (done.load(std::memory_order_acquire)) return PMC_OK;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "%s: cannot reserve %zu bytes of LDS: %s", what, bytes, hipGetErrorString(e));
  done.store(true, std::memory_order_release);
  return PMC_OK;
}

struct GemmArgs {
  int dtype = PMC_BF16;
  bool trans_a = false, trans_b = false;
  int M = 0, N = 0, K = 0;
  const void* A = nullptr;
  int lda = 0;
  const void* B = nullptr;
  int ldb = 0;
  void* C = nullptr;
  int ldc = 0;
  int epilogue = PMC_EPI_NONE;
  const void* bias = nullptr;   // [N], storage type
  const void* resid = nullptr;  // [M, N], pitch ldc
  void* aux = nullptr;          // [M, N], pitch ldc
  void* ws = nullptr;           // optional scratch for split-K partial products (256-byte aligned)
  size_t ws_bytes = 0;
};

// Weight gradients of several queued microbatches as ONE product: C[M,N] (fp32) += sum_i A_i^T . B_i
// with A_i stored [K,M] (pitch lda) and B_i stored [K,N] (pitch ldb), bf16.  K a multiple of 64.
struct GroupedWgradArgs {
  int M = 0, N = 0, K = 0;  // K of ONE piece
  int count = 0;            // 1 .. PMC_MAX_QUEUED_W pieces
  const void* A[PMC_MAX_QUEUED_W] = {};
  const void* B[PMC_MAX_QUEUED_W] = {};
  int lda = 0, ldb = 0;
  float* C = nullptr;
  int ldc = 0;
};
int gemm_bf16_grouped_wgrad(hipStream_t stream, const GroupedWgradArgs& a);

// Scratch a product of this shape can use (0: none).
size_t gemm_scratch_bytes(int dtype, int M, int N, int K);

int gemm(hipStream_t stream, const GemmArgs& a);
int gemm_f32(hipStream_t stream, const GemmArgs& a);
int gemm_bf16(hipStream_t stream, const GemmArgs& a);

int layernorm_forward(hipStream_t stream, int dtype, int rows, int h, const void* x, const void* gain,
                      const void* bias, float eps, void* y, float* mean, float* rstd, void* x_copy);
// partial: fp32 scratch of layernorm_backward_scratch_floats(rows, h) floats.  The kernel leaves one
// row of gain/bias-gradient partial sums per workgroup there; a second, tiny kernel adds them into
// dgain/dbias.  With `defer` given that second step is only noted down (the scratch must then stay
// untouched, one region per call) and layernorm_backward_reduce runs all noted reductions in ONE
// launch: a backward pass has two LayerNorms per layer and pays for one such launch, not for 2 L.
struct LnPartialJobs {
  static constexpr int kMax = 16;
  const float* partial[kMax];
  float* dgain[kMax];
  float* dbias[kMax];
  int parts[kMax];
  int count = 0;
};
size_t layernorm_backward_scratch_floats(int rows, int h);
int layernorm_backward(hipStream_t stream, int dtype, int rows, int h, const void* dy, const void* x,
                       const void* gain, const float* mean, const float* rstd, const void* resid, void* dx,
                       float* dgain, float* dbias, float* partial, LnPartialJobs* defer = nullptr);
int layernorm_backward_reduce(hipStream_t stream, int h, const LnPartialJobs& jobs);
// As layernorm_backward with the partial sums in a device array built into the library (no workspace,
// no allocation); PMC_ERR_NOMEM when layernorm_backward_scratch_floats(rows, h) floats do not fit in
// layernorm_backward_static_scratch_bytes().
size_t layernorm_backward_static_scratch_bytes();
int layernorm_backward_static(hipStream_t stream, int dtype, int rows, int h, const void* dy, const void* x,
                              const void* gain, const float* mean, const float* rstd, const void* resid, void* dx,
                              float* dgain, float* dbias);

int attention_forward(hipStream_t stream, int dtype, int batch, int seq, int heads, int head_dim, int causal,
                      const void* qkv, void* o, float* lse);
// scratch: dq staging [batch*seq, heads*head_dim] in the storage type, then delta fp32 [batch, heads, seq].
size_t attention_backward_scratch_bytes(int dtype, int batch, int seq, int heads, int head_dim);
int attention_backward(hipStream_t stream, int dtype, int batch, int seq, int heads, int head_dim, int causal,
                       const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                       void* scratch);

// out[c] += sum over rows of a[row][c] (fp32 out), for up to four matrices of `rows` rows in one
// launch; first_block is filled in by column_sums.
struct ColumnSumJobs {
  const void* a[4];
  float* out[4];
  int n[4];
  int lda[4];
  int first_block[5];
  int count;
};
int column_sums(hipStream_t stream, int dtype, int rows, ColumnSumJobs jobs);
int column_sum(hipStream_t stream, int dtype, int rows, int n, const void* a, int lda, float* out);

int copy_rows(hipStream_t stream, int dtype, int rows, int cols, const void* src, int ld_src, void* dst, int ld_dst);

}  // namespace k
}  // namespace pmc
