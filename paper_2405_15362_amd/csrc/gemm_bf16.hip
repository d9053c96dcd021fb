// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate) for the
// projections of the three passes:
//   F: Y  = X . W  (+ bias, + residual, GeLU)      A stored [M,K], B stored [K,N]
//   B: dX = dY . W^T  (* GeLU')                    A stored [M,K], B stored [N,K]
//   W: dW += X^T . dY  (fp32 accumulate)           A stored [K,M], B stored [K,N]
// A workgroup computes a BM x BN tile; operand tiles go global -> registers -> LDS (double
// buffered, one barrier per K step) and are read back as MFMA fragments.  An operand whose
// contraction index is contiguous in memory is read with 16-byte LDS loads; one whose contraction
// index is the slow dimension is kept in its natural layout in LDS and read with the transposing
// load ds_read_b64_tr_b16, so no operand is ever transposed in HBM.  The MFMA is issued with the
// operand roles exchanged (B-fragment as first operand), which leaves every lane with four
// consecutive output columns of one row and lets the epilogue use 8/16-byte accesses.
// Workgroup ids are remapped so that the ids resident on one XCD (they are dealt round-robin over
// the 8 XCDs) cover a compact group of tiles and share operand panels in that XCD's L2.
#include "dev_common.h"
#include "kernels.h"

namespace pmc {
namespace k {
namespace {

struct GemmParams {
  const bf16_t* A;
  const bf16_t* B;
  void* C;
  const bf16_t* bias;
  const bf16_t* resid;
  bf16_t* aux;
  int M, N, K, lda, ldb, ldc;
  int tiles_m, tiles_n;
};

constexpr int kPadK = 8;    // K-major tile: row pitch BK + 8 elements (144 B for BK = 64)
constexpr int kPadMN = 32;  // MN-major tile: row pitch ROWS + 32 elements (pitch = 64 mod 256 bytes)

template <int ROWS, int BK, bool KMAJ>
struct Tile {
  static constexpr int pitch = KMAJ ? BK + kPadK : ROWS + kPadMN;
  static constexpr int elems = KMAJ ? ROWS * pitch : BK * pitch;
};

// Global -> register staging of one operand tile: CH 16-byte chunks per thread.
template <int ROWS, int BK, bool KMAJ, int NT>
struct Stager {
  static constexpr int CH = ROWS * BK / 8 / NT;
  static_assert(ROWS * BK / 8 % NT == 0, "tile must split evenly over the threads");
  u32x4 r[CH];

  __device__ __forceinline__ void load(const bf16_t* __restrict__ base, int ld, int mn0, int k0, int mn_total, int K,
                                       int tid) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * NT;
      int mn, kk;
      if (KMAJ) {
        mn = c / (BK / 8);
        kk = (c % (BK / 8)) * 8;
      } else {
        kk = c / (ROWS / 8);
        mn = (c % (ROWS / 8)) * 8;
      }
      const bool ok = (mn0 + mn < mn_total) && (k0 + kk < K);
      const size_t off = KMAJ ? (size_t)(mn0 + mn) * ld + (k0 + kk) : (size_t)(k0 + kk) * ld + (mn0 + mn);
      u32x4 z = {0u, 0u, 0u, 0u};
      r[i] = ok ? *reinterpret_cast<const u32x4*>(base + off) : z;
    }
  }
  __device__ __forceinline__ void store(bf16_t* lds, int tid) const {
    constexpr int pitch = Tile<ROWS, BK, KMAJ>::pitch;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * NT;
      int off;
      if (KMAJ) off = (c / (BK / 8)) * pitch + (c % (BK / 8)) * 8;
      else off = (c / (ROWS / 8)) * pitch + (c % (ROWS / 8)) * 8;
      *reinterpret_cast<u32x4*>(lds + off) = r[i];
    }
  }
};

// MFMA operand fragment for 32 rows starting at r0 and 16 contraction indices starting at ks:
// lane l holds row r0 + l%32, contraction indices ks + 8*(l/32) .. +7.
template <int ROWS, int BK, bool KMAJ>
__device__ __forceinline__ bf16x8 read_frag(const bf16_t* lds, int r0, int ks, int lane) {
  constexpr int pitch = Tile<ROWS, BK, KMAJ>::pitch;
  if (KMAJ) {
    return *reinterpret_cast<const bf16x8*>(lds + (r0 + (lane & 31)) * pitch + ks + 8 * (lane >> 5));
  } else {
    // ds_read_b64_tr_b16 works on groups of 16 lanes: lane j of a group supplies the address of 4
    // consecutive elements of row j/4 (piece j%4 of a 16-element span) and receives the 4 rows of
    // column j.  Groups 0..3 of the wave cover (columns 0-15 | 16-31) x (k 0-7 | 8-15).
    const int g = lane >> 4, j = lane & 15;
    const bf16_t* p = lds + (ks + 8 * (g >> 1) + (j >> 2)) * pitch + r0 + 16 * (g & 1) + 4 * (j & 3);
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * pitch));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
}

__device__ __forceinline__ void unpack4(u32x2 v, float* f) {
  f[0] = bf16lo_to_f32(v[0]); f[1] = bf16hi_to_f32(v[0]); f[2] = bf16lo_to_f32(v[1]); f[3] = bf16hi_to_f32(v[1]);
}
__device__ __forceinline__ u32x2 pack4(const float* f) {
  u32x2 v = {pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3])};
  return v;
}

template <int BM, int BN, int BK, int WM, int WN, bool A_KMAJ, bool B_KMAJ, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_kernel(GemmParams p) {
  constexpr int WAVES_N = BN / WN;
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int TM = WM / 32, TN = WN / 32;
  using TileA = Tile<BM, BK, A_KMAJ>;
  using TileB = Tile<BN, BK, B_KMAJ>;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  constexpr int kStage = TileA::elems + TileB::elems;  // one buffer: A tile then B tile

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  // Workgroup id -> tile.  Ids are dealt round-robin over 8 XCDs; give each XCD a contiguous run
  // of tile indices, then walk tiles in column groups 8 tiles of M tall.
  const int ntiles = p.tiles_m * p.tiles_n;
  int pid = blockIdx.x;
  {
    const int xcd = pid & 7, local = pid >> 3, lo = ntiles >> 3, rem = ntiles & 7;
    pid = xcd * lo + (xcd < rem ? xcd : rem) + local;
  }
  constexpr int GROUP = 8;
  const int per_group = GROUP * p.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GROUP;
  const int group_m = min(p.tiles_m - first_m, GROUP);
  const int tile_m = first_m + (pid % per_group) % group_m;
  const int tile_n = (pid % per_group) / group_m;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  Stager<BM, BK, A_KMAJ, NT> sa;
  Stager<BN, BK, B_KMAJ, NT> sb;
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (p.K + BK - 1) / BK;
  sa.load(p.A, p.lda, m0, 0, p.M, p.K, tid);
  sb.load(p.B, p.ldb, n0, 0, p.N, p.K, tid);
  sa.store(smem, tid);
  sb.store(smem + TileA::elems, tid);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const bf16_t* cur_a = smem + (kt & 1) * kStage;
    const bf16_t* cur_b = cur_a + TileA::elems;
    if (kt + 1 < nk) {
      sa.load(p.A, p.lda, m0, (kt + 1) * BK, p.M, p.K, tid);
      sb.load(p.B, p.ldb, n0, (kt + 1) * BK, p.N, p.K, tid);
    }
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = read_frag<BM, BK, A_KMAJ>(cur_a, wm0 + 32 * i, ks, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = read_frag<BN, BK, B_KMAJ>(cur_b, wn0 + 32 * j, ks, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      bf16_t* nxt = smem + ((kt + 1) & 1) * kStage;
      sa.store(nxt, tid);
      sb.store(nxt + TileA::elems, tid);
    }
    __syncthreads();
  }

  // Epilogue.  acc[i][j][r]: row m = m0 + wm0 + 32 i + lane%32, column
  // n = n0 + wn0 + 32 j + 8 (r/4) + 4 (lane/32) + r%4.
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm0 + 32 * i + (lane & 31);
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn0 + 32 * j + 8 * q + 4 * (lane >> 5);
        if (n >= p.N) continue;
        const size_t idx = (size_t)m * p.ldc + n;
        float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        if (EPI == PMC_EPI_ACCUM_F32) {
          float* c = reinterpret_cast<float*>(p.C) + idx;
          f32x4 old = *reinterpret_cast<f32x4*>(c);
          f32x4 out = {old[0] + v[0], old[1] + v[1], old[2] + v[2], old[3] + v[3]};
          *reinterpret_cast<f32x4*>(c) = out;
          continue;
        }
        bf16_t* c = reinterpret_cast<bf16_t*>(p.C) + idx;
        if (EPI == PMC_EPI_BIAS || EPI == PMC_EPI_BIAS_RESID || EPI == PMC_EPI_BIAS_GELU) {
          float b[4];
          unpack4(*reinterpret_cast<const u32x2*>(p.bias + n), b);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += b[e];
        }
        if (EPI == PMC_EPI_BIAS_RESID) {
          float r[4];
          unpack4(*reinterpret_cast<const u32x2*>(p.resid + idx), r);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += r[e];
        }
        if (EPI == PMC_EPI_DGELU) {
          float u[4];
          unpack4(*reinterpret_cast<const u32x2*>(p.aux + idx), u);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_f(u[e]);
        }
        *reinterpret_cast<u32x2*>(c) = pack4(v);
        if (EPI == PMC_EPI_BIAS_GELU) {
          float g[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) g[e] = gelu_f(v[e]);
          *reinterpret_cast<u32x2*>(p.aux + idx) = pack4(g);
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN, bool A_KMAJ, bool B_KMAJ, int EPI>
int launch(hipStream_t st, GemmParams p) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr size_t lds = 2 * sizeof(bf16_t) * (Tile<BM, BK, A_KMAJ>::elems + Tile<BN, BK, B_KMAJ>::elems);
  static_assert(lds <= 160 * 1024, "tile does not fit the 160 KB LDS");
  auto kern = gemm_bf16_kernel<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, EPI>;
  static bool configured = false;  // per instantiation
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return fail(PMC_ERR_HIP, "gemm_bf16: cannot reserve %zu bytes of LDS: %s", lds, hipGetErrorString(e));
    configured = true;
  }
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  kern<<<dim3(p.tiles_m * p.tiles_n), dim3(NT), lds, st>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "gemm_bf16 launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

template <int BM, int BN, int BK, int WM, int WN, bool A_KMAJ, bool B_KMAJ>
int launch_epi(hipStream_t st, const GemmParams& p, int epi) {
  switch (epi) {
    case PMC_EPI_NONE: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_NONE>(st, p);
    case PMC_EPI_BIAS: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_BIAS>(st, p);
    case PMC_EPI_BIAS_RESID: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_BIAS_RESID>(st, p);
    case PMC_EPI_BIAS_GELU: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_BIAS_GELU>(st, p);
    case PMC_EPI_DGELU: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_DGELU>(st, p);
    case PMC_EPI_ACCUM_F32: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_ACCUM_F32>(st, p);
  }
  return fail(PMC_ERR_INVALID, "gemm_bf16: unknown epilogue %d", epi);
}

template <bool A_KMAJ, bool B_KMAJ>
int launch_tile(hipStream_t st, const GemmParams& p, int epi) {
  // Large tile when it still yields at least about one workgroup per compute unit.
  const long big_tiles = (long)((p.M + 255) / 256) * ((p.N + 255) / 256);
  if (big_tiles >= 200) return launch_epi<256, 256, 64, 128, 128, A_KMAJ, B_KMAJ>(st, p, epi);
  return launch_epi<128, 128, 64, 64, 64, A_KMAJ, B_KMAJ>(st, p, epi);
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

int gemm_bf16(hipStream_t st, const GemmArgs& a) {
  if (a.M % 8 || a.N % 8 || a.K % 8) return fail(PMC_ERR_INVALID, "gemm_bf16: M=%d N=%d K=%d must be multiples of 8", a.M, a.N, a.K);
  if (a.lda % 8 || a.ldb % 8 || a.ldc % 4) return fail(PMC_ERR_INVALID, "gemm_bf16: pitches must be multiples of 8 (lda=%d ldb=%d ldc=%d)", a.lda, a.ldb, a.ldc);
  if (!aligned(a.A, 16) || !aligned(a.B, 16) || !aligned(a.C, 16) || (a.bias && !aligned(a.bias, 8)) ||
      (a.resid && !aligned(a.resid, 8)) || (a.aux && !aligned(a.aux, 8)))
    return fail(PMC_ERR_INVALID, "gemm_bf16: operands must be 16-byte aligned");
  GemmParams p;
  p.A = (const bf16_t*)a.A; p.B = (const bf16_t*)a.B; p.C = a.C;
  p.bias = (const bf16_t*)a.bias; p.resid = (const bf16_t*)a.resid; p.aux = (bf16_t*)a.aux;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc;
  p.tiles_m = p.tiles_n = 0;
  const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
  if (a_kmaj && b_kmaj) return launch_tile<true, true>(st, p, a.epilogue);
  if (a_kmaj && !b_kmaj) return launch_tile<true, false>(st, p, a.epilogue);
  if (!a_kmaj && b_kmaj) return launch_tile<false, true>(st, p, a.epilogue);
  return launch_tile<false, false>(st, p, a.epilogue);
}

}  // namespace k
}  // namespace pmc
