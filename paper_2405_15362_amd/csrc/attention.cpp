// Chooses the attention kernels for a storage type and checks the shapes they assume.
#include "kernels.h"

namespace pmc {
namespace k {

int attention_forward_simple(hipStream_t st, int dtype, int batch, int seq, int heads, int dh, int causal,
                             const void* qkv, void* o, float* lse);
int attention_backward_simple(hipStream_t st, int dtype, int batch, int seq, int heads, int dh, int causal,
                              const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                              void* dq_stage, float* delta);

int attention_forward_mfma(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv, void* o,
                           float* lse);
int attention_backward_mfma(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv,
                            const void* o, const float* lse, const void* d_o, void* dqkv, void* dq_stage, float* delta);

namespace {
// bf16 storage with a head size that is a multiple of 8 (up to 128) runs on the matrix cores;
// everything else (fp32 mode, other head sizes) on the plain-arithmetic kernels.
bool use_mfma(int dtype, int head_dim) { return dtype == PMC_BF16 && head_dim >= 8 && head_dim <= 128 && head_dim % 8 == 0; }
size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
size_t elem(int dtype) { return dtype == PMC_F32 ? 4 : 2; }
}  // namespace

int attention_forward(hipStream_t st, int dtype, int batch, int seq, int heads, int head_dim, int causal,
                      const void* qkv, void* o, float* lse) {
  if (!qkv || !o || !lse) return fail(PMC_ERR_INVALID, "attention_forward: NULL pointer");
  if (dtype != PMC_F32 && dtype != PMC_BF16) return fail(PMC_ERR_INVALID, "attention_forward: bad dtype %d", dtype);
  if (use_mfma(dtype, head_dim)) return attention_forward_mfma(st, batch, seq, heads, head_dim, causal, qkv, o, lse);
  return attention_forward_simple(st, dtype, batch, seq, heads, head_dim, causal, qkv, o, lse);
}

size_t attention_backward_scratch_bytes(int dtype, int batch, int seq, int heads, int head_dim) {
  const size_t tokens = (size_t)batch * seq;
  return align256(tokens * heads * head_dim * elem(dtype)) + align256(tokens * heads * sizeof(float));
}

int attention_backward(hipStream_t st, int dtype, int batch, int seq, int heads, int head_dim, int causal,
                       const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv, void* scratch) {
  if (!qkv || !o || !lse || !d_o || !dqkv || !scratch) return fail(PMC_ERR_INVALID, "attention_backward: NULL pointer");
  if (dtype != PMC_F32 && dtype != PMC_BF16) return fail(PMC_ERR_INVALID, "attention_backward: bad dtype %d", dtype);
  const size_t tokens = (size_t)batch * seq;
  const int h = heads * head_dim;
  const int vec = dtype == PMC_F32 ? 4 : 8;
  if (h % vec) return fail(PMC_ERR_INVALID, "attention_backward: hidden %d must be a multiple of %d", h, vec);
  char* dq_stage = (char*)scratch;
  float* delta = (float*)(dq_stage + align256(tokens * h * elem(dtype)));
  // dq goes to the staging buffer because q is still needed by the dk/dv kernel, which reads k, v
  // from qkv and writes dk, dv to the same columns of dqkv (dqkv may be qkv itself: a key tile is
  // read only by the workgroup that later overwrites it).
  const int rc = use_mfma(dtype, head_dim)
                     ? attention_backward_mfma(st, batch, seq, heads, head_dim, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta)
                     : attention_backward_simple(st, dtype, batch, seq, heads, head_dim, causal, qkv, o, lse, d_o, dqkv,
                                                 dq_stage, delta);
  if (rc) return rc;
  return copy_rows(st, dtype, (int)tokens, h, dq_stage, h, dqkv, 3 * h);
}

}  // namespace k
}  // namespace pmc
