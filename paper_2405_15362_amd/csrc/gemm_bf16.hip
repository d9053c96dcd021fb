// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate) for the
// projections of the three passes:
//   F: Y  = X . W  (+ bias, + residual, GeLU)      A stored [M,K], B stored [K,N]
//   B: dX = dY . W^T  (* GeLU')                    A stored [M,K], B stored [N,K]
//   W: dW += X^T . dY  (fp32 accumulate)           A stored [K,M], B stored [K,N]
// Two kernels share the fragment layouts and the epilogue:
//
//  * gemm_bf16_dma_kernel, the fast path (K a multiple of 64).  Operand tiles go straight from
//    global memory into LDS (buffer_load ... lds, no registers in between) into a ring of 2 or 3
//    stages; rows past the edge are clamped, never branched on.  LDS tiles are unpadded and
//    XOR-swizzled in 16-byte chunks so that both the DMA writes and the fragment reads are free of
//    bank conflicts.  The K loop is software pipelined by hand: while the MFMAs of one 16-wide K
//    step run, the fragments of the next step are read from LDS into a second register set, in a
//    fixed interleave; the barrier that releases a stage sits before the last K step of a tile, so
//    the first fragments of the next tile are read under that step's MFMAs and no LDS latency is
//    exposed at tile boundaries.  The DMA loads are issued as inline assembly and waited for with
//    explicit vmcnt values, because the compiler would otherwise drain every outstanding load
//    before each LDS read.
//  * gemm_bf16_kernel, the general path (any K multiple of 8, all layout/epilogue combinations):
//    global -> registers -> padded LDS tiles, double buffered.
//
// An operand whose contraction index is contiguous in memory is read from LDS with 16-byte loads;
// one whose contraction index is the slow dimension (W in F; X and dY in W) keeps its natural
// layout in LDS and is read with the transposing load ds_read_b64_tr_b16, so no operand is ever
// transposed in HBM.  The MFMA is issued with the operand roles exchanged (B-fragment as first
// operand), which leaves every lane with four consecutive output columns of one row and lets the
// epilogue use 8/16-byte accesses.  Workgroup ids are remapped so that the ids resident on one XCD
// (they are dealt round-robin over the 8 XCDs) cover a compact group of tiles and share operand
// panels in that XCD's L2.
#include <cstdlib>

#include "dev_common.h"
#include "kernels.h"

namespace pmc {
namespace k {
namespace {

constexpr int kMaxSegments = PMC_MAX_QUEUED_W;

struct GemmParams {
  const bf16_t* A;
  const bf16_t* B;
  void* C;
  const bf16_t* bias;
  const bf16_t* resid;
  bf16_t* aux;
  int M, N, K, lda, ldb, ldc;
  int tiles_m, tiles_n;
  int group_m;            // height, in tiles, of the column groups the tiles are walked in (see tile_of_pid)
  int k_tiles_per_split;  // fast path: 64-wide K tiles each blockIdx.y handles (all of K when not split)
  // Segmented contraction (weight gradients of several queued microbatches in one product): the K
  // axis is the concatenation of nseg pieces of seg_tiles 64-wide tiles each, piece i living at
  // (Aseg[i], Bseg[i]) with the pitches lda, ldb.  nseg = 0: one piece at (A, B).
  const bf16_t* Aseg[kMaxSegments];
  const bf16_t* Bseg[kMaxSegments];
  int nseg, seg_tiles;
};

constexpr int kEpiPartial = 100;  // fast path, split K: store the fp32 partial product of split blockIdx.y

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

// Applies epilogue EPI to four consecutive output columns n .. n+3 of row m and stores them.
template <int EPI>
__device__ __forceinline__ void store_quad(const GemmParams& p, float (&v)[4], int m, int n) {
  const size_t idx = (size_t)m * p.ldc + n;
  if (EPI == kEpiPartial) {
    float* c = reinterpret_cast<float*>(p.C) + (size_t)blockIdx.y * p.M * p.N + (size_t)m * p.N + n;
    f32x4 out = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4*>(c) = out;
    return;
  }
  if (EPI == PMC_EPI_ACCUM_F32) {
    float* c = reinterpret_cast<float*>(p.C) + idx;
    f32x4 old = *reinterpret_cast<f32x4*>(c);
    f32x4 out = {old[0] + v[0], old[1] + v[1], old[2] + v[2], old[3] + v[3]};
    *reinterpret_cast<f32x4*>(c) = out;
    return;
  }
  bf16_t* c = reinterpret_cast<bf16_t*>(p.C) + idx;
  if (EPI == PMC_EPI_BIAS || EPI == PMC_EPI_BIAS_RESID || EPI == PMC_EPI_BIAS_GELU || EPI == PMC_EPI_BIAS_GELU_GRAD) {
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
    for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_fast(u[e]);
  }
  if (EPI == PMC_EPI_MUL) {
    float u[4];
    unpack4(*reinterpret_cast<const u32x2*>(p.aux + idx), u);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= u[e];
  }
  if (EPI == PMC_EPI_BIAS_GELU_GRAD) {
    float g[4], dg[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) gelu_both_fast(v[e], g[e], dg[e]);
    *reinterpret_cast<u32x2*>(c) = pack4(dg);
    *reinterpret_cast<u32x2*>(p.aux + idx) = pack4(g);
    return;
  }
  *reinterpret_cast<u32x2*>(c) = pack4(v);
  if (EPI == PMC_EPI_BIAS_GELU) {
    float g[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) g[e] = gelu_fast(v[e]);
    *reinterpret_cast<u32x2*>(p.aux + idx) = pack4(g);
  }
}

// Epilogue shared by both kernels.  acc[i][j][r] of a wave whose tile starts at (mw0, nw0): row
// m = mw0 + 32 i + lane%32, columns n = nw0 + 32 j + 8 (r/4) + 4 (lane/32) + r%4.
template <int TM, int TN, int EPI>
__device__ __forceinline__ void epilogue(const GemmParams& p, f32x16 (&acc)[TM][TN], int mw0, int nw0, int lane) {
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = mw0 + 32 * i + (lane & 31);
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = nw0 + 32 * j + 8 * q + 4 * (lane >> 5);
        if (n >= p.N) continue;
        float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        store_quad<EPI>(p, v, m, n);
      }
    }
  }
}

__device__ __forceinline__ void unpack8(u32x4 v, float* f) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = bf16lo_to_f32(v[e]);
    f[2 * e + 1] = bf16hi_to_f32(v[e]);
  }
}
__device__ __forceinline__ u32x4 pack8(const float* f) {
  u32x4 v = {pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7])};
  return v;
}

// What an epilogue reads besides the bias for eight consecutive output columns: the old fp32 sums
// (ACCUM), the residual (BIAS_RESID) or the GeLU input (DGELU).  Fetched ahead of use, a whole
// 32-row slab at a time, so that many loads are in flight per wave.
template <int EPI>
struct OctOperand {
  f32x4 lo, hi;  // ACCUM
  u32x4 packed;  // BIAS_RESID, DGELU
  static constexpr bool used =
      EPI == PMC_EPI_ACCUM_F32 || EPI == PMC_EPI_BIAS_RESID || EPI == PMC_EPI_DGELU || EPI == PMC_EPI_MUL;
  __device__ __forceinline__ void load(const GemmParams& p, int m, int n) {
    const size_t idx = (size_t)m * p.ldc + n;
    if (EPI == PMC_EPI_ACCUM_F32) {
      // streamed once: keep the fp32 sums out of the way of the operand panels in L2
      const float* c = reinterpret_cast<const float*>(p.C) + idx;
      lo = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(c));
      hi = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(c + 4));
    } else if (EPI == PMC_EPI_BIAS_RESID) {
      packed = *reinterpret_cast<const u32x4*>(p.resid + idx);
    } else if (EPI == PMC_EPI_DGELU || EPI == PMC_EPI_MUL) {
      packed = *reinterpret_cast<const u32x4*>(p.aux + idx);
    }
  }
};

// Applies epilogue EPI to eight consecutive output columns n .. n+7 of row m and stores them
// (16 bytes per lane for bf16 results, 32 for fp32 ones).  Same arithmetic as store_quad.
template <int EPI>
__device__ __forceinline__ void store_oct(const GemmParams& p, float (&v)[8], int m, int n, const OctOperand<EPI>& x) {
  const size_t idx = (size_t)m * p.ldc + n;
  if (EPI == kEpiPartial || EPI == PMC_EPI_ACCUM_F32) {
    float* c = EPI == kEpiPartial
                   ? reinterpret_cast<float*>(p.C) + (size_t)blockIdx.y * p.M * p.N + (size_t)m * p.N + n
                   : reinterpret_cast<float*>(p.C) + idx;
    f32x4 lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
    if (EPI == PMC_EPI_ACCUM_F32) {
      lo = x.lo + lo;
      hi = x.hi + hi;
      __builtin_nontemporal_store(lo, reinterpret_cast<f32x4*>(c));
      __builtin_nontemporal_store(hi, reinterpret_cast<f32x4*>(c + 4));
      return;
    }
    *reinterpret_cast<f32x4*>(c) = lo;
    *reinterpret_cast<f32x4*>(c + 4) = hi;
    return;
  }
  if (EPI == PMC_EPI_BIAS || EPI == PMC_EPI_BIAS_RESID || EPI == PMC_EPI_BIAS_GELU || EPI == PMC_EPI_BIAS_GELU_GRAD) {
    float b[8];
    unpack8(*reinterpret_cast<const u32x4*>(p.bias + n), b);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += b[e];
  }
  if (EPI == PMC_EPI_BIAS_RESID) {
    float r[8];
    unpack8(x.packed, r);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += r[e];
  }
  if (EPI == PMC_EPI_DGELU) {
    float u[8];
    unpack8(x.packed, u);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_fast(u[e]);
  }
  if (EPI == PMC_EPI_MUL) {
    float u[8];
    unpack8(x.packed, u);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= u[e];
  }
  if (EPI == PMC_EPI_BIAS_GELU_GRAD) {
    float g[8], dg[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) gelu_both_fast(v[e], g[e], dg[e]);
    *reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(p.C) + idx) = pack8(dg);
    *reinterpret_cast<u32x4*>(p.aux + idx) = pack8(g);
    return;
  }
  *reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(p.C) + idx) = pack8(v);
  if (EPI == PMC_EPI_BIAS_GELU) {
    float g[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] = gelu_fast(v[e]);
    *reinterpret_cast<u32x4*>(p.aux + idx) = pack8(g);
  }
}

// Epilogue of the fast path.  In the accumulator layout a store instruction would touch 32 rows
// with 16 bytes each; instead each wave passes its tile, 32 rows at a time, through a private
// LDS slab [32][32 TN + 4] of fp32 and reads it back with 8 consecutive columns per lane, so a
// store instruction covers whole 128-byte (bf16) or 256-byte (fp32) row segments.  The pitch of
// 32 TN + 4 words spreads both the column-quad writes and the row-major reads over all banks.
// Only the wave itself touches its slab: LDS operations of one wave complete in order, so no
// barrier is needed between the passes.
// J0, JN: the column tiles J0 .. J0 + JN - 1 of the wave's TN are staged (JN a power of two, so that
// whole rows divide a wave's 64 lanes); a tile that is 5 wide goes out as 4 + 1.
template <int TM, int TN, int EPI, int J0 = 0, int JN = TN>
__device__ __forceinline__ void epilogue_staged(const GemmParams& p, f32x16 (&acc)[TM][TN], float* slab, int mw0,
                                                int nw0_wave, int lane) {
  static_assert((JN & (JN - 1)) == 0 && JN <= 8 && J0 + JN <= TN, "column group");
  constexpr int WN = 32 * JN, PITCH = WN + 4;
  const int nw0 = nw0_wave + 32 * J0;
  constexpr int LPR = WN / 8;     // lanes per row on the way out
  constexpr int RPP = 64 / LPR;   // rows per pass
  constexpr int NPASS = 32 / RPP;
  const int orow = lane / LPR, ocol = 8 * (lane % LPR);
  const int n = nw0 + ocol;
  // operands of slab i + 1 are requested before slab i is staged and stored
  OctOperand<EPI> ahead[2][NPASS];
  auto fetch = [&](int i, OctOperand<EPI> (&dst)[NPASS]) {
    if (!OctOperand<EPI>::used) return;
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int m = mw0 + 32 * i + pass * RPP + orow;
      if (m < p.M && n < p.N) dst[pass].load(p, m, n);
    }
  };
  fetch(0, ahead[0]);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (i + 1 < TM) fetch(i + 1, ahead[(i + 1) & 1]);
#pragma unroll
    for (int j = 0; j < JN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 t = {acc[i][J0 + j][4 * q], acc[i][J0 + j][4 * q + 1], acc[i][J0 + j][4 * q + 2], acc[i][J0 + j][4 * q + 3]};
        *reinterpret_cast<f32x4*>(slab + (lane & 31) * PITCH + 32 * j + 8 * q + 4 * (lane >> 5)) = t;
      }
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int row = pass * RPP + orow;
      const f32x4 lo = *reinterpret_cast<const f32x4*>(slab + row * PITCH + ocol);
      const f32x4 hi = *reinterpret_cast<const f32x4*>(slab + row * PITCH + ocol + 4);
      const int m = mw0 + 32 * i + row;
      if (m < p.M && n < p.N) {
        float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        store_oct<EPI>(p, v, m, n, ahead[i & 1][pass]);
      }
    }
  }
}

// Second half of a split-K product: adds the fp32 partials of the splits in ascending order (a
// fixed order, so the result does not depend on scheduling) and applies the epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmParams p, const float* __restrict__ partial, int splits) {
#if defined(__HIP_DEVICE_COMPILE__)
  const size_t quad = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t e0 = quad * 4, total = (size_t)p.M * p.N;
  if (e0 >= total) return;
  const int m = (int)(e0 / p.N), n = (int)(e0 % p.N);
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(partial + (size_t)s * total + e0);
    v[0] += t[0]; v[1] += t[1]; v[2] += t[2]; v[3] += t[3];
  }
  store_quad<EPI>(p, v, m, n);
#endif
}

// Workgroup id -> (tile_m, tile_n).  Ids are dealt round-robin over 8 XCDs; give each XCD a
// contiguous run of tile indices, then walk tiles in column groups group_m tiles of M tall.  The 32
// tiles an XCD works on at a time are then a block of group_m x 32/group_m tiles, whose operand
// panels (group_m BM rows of A, 32/group_m BN rows of B per K step) are what that XCD's L2 has to
// fetch.  Measured on whole steps: 4 for the 256-row tiles (+1 % at hidden 4096 over 8, nothing at
// 5120), 8 for the smaller ones (4 costs the 64 x 128 products 2 %).  The gemm_group tuning switch forces a height.
__device__ __forceinline__ void tile_of_pid(const GemmParams& p, int pid, int& tile_m, int& tile_n) {
  const int ntiles = p.tiles_m * p.tiles_n;
  const int xcd = pid & 7, local = pid >> 3, lo = ntiles >> 3, rem = ntiles & 7;
  pid = xcd * lo + (xcd < rem ? xcd : rem) + local;
  const int GROUP = p.group_m;
  const int per_group = GROUP * p.tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GROUP;
  const int group_m = min(p.tiles_m - first_m, GROUP);
  tile_m = first_m + (pid % per_group) % group_m;
  tile_n = (pid % per_group) / group_m;
}
__device__ __forceinline__ void tile_of_block(const GemmParams& p, int& tile_m, int& tile_n) {
  tile_of_pid(p, blockIdx.x, tile_m, tile_n);
}

// ---------------------------------------------------------------------------------------------
// Fast path: direct-to-LDS operand tiles, swizzled, hand-pipelined.
//
// LDS tile layouts (BK = 64, no padding; a "chunk" is 16 bytes = 8 elements):
//   contraction-contiguous operand: [rows][64]; chunk position p of row r holds k-chunk
//       p ^ ((r >> 1) & 7)   -> 16 lanes reading 16 consecutive rows at one k hit 16 distinct
//       16-byte bank groups;
//   other operand: [64 k][ROWS]; chunk position p of k-row kr holds chunk p ^ kswz(kr) = p ^ ((kr & 3) << 2)
//       -> the four k-rows one half-wave touches in a transposing read fall into four different
//       64-byte bank quarters.
// One buffer_load...lds instruction of a wave fills 1 KB of LDS (lane l writes bytes 16 l .. 16 l + 15
// of it), so the swizzle is applied to the GLOBAL address each lane fetches from.
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// Chunk swizzle of k-row kr in a [64 k][ROWS] tile.  A k-row of 128 n rows (a multiple of 256 bytes)
// starts in the same bank as its neighbours, so the four k-rows of a transposing read are moved to
// four different 64-byte quarters by their two low bits.  In a 320-row tile (640 bytes per k-row)
// consecutive k-rows already sit 128 bytes apart; bit 1 of kr supplies the other 64 bytes, and
// flipping only bit 2 of the chunk index keeps every chunk inside its own group of 8 (320 / 8 = 40
// chunks per k-row is not a multiple of 16).
template <int ROWS>
__device__ __forceinline__ constexpr int kswz(int kr) {
  return ROWS % 128 == 0 ? ((kr & 3) << 2) : (((kr >> 1) & 1) << 2);
}

// BK: K rows of the tile; 64 everywhere except the [32 k][ROWS] tiles of the two-workgroup weight-gradient kernel
// (the [rows][64] layout's swizzle is defined for 64 only).
template <int ROWS, bool KMAJ, int NW, int BK = 64>
struct DmaLoader {
  static constexpr int NL = ROWS * BK * 2 / 1024 / NW;  // 1 KB loads per wave per tile
  static_assert(ROWS * BK * 2 / 1024 % NW == 0, "tile must split evenly over the waves");
  static_assert(BK == 64 || (!KMAJ && BK == 32), "K depth of a tile");
  static_assert(KMAJ || ROWS % 128 == 0 || ROWS == 320, "the [64 k][rows] swizzle is defined for whole 128-row groups and for 320 rows");
  uint32_t voff[NL];  // byte offset of this lane's chunk at K offset 0

  // Wave w issues loads w*NL .. w*NL+NL-1; load q fills tile bytes [1024 q, 1024 q + 1024).
  // Rows (or columns) past the edge of the matrix are clamped to the last valid ones: what they
  // produce lands in output rows/columns that the epilogue does not store.
  __device__ __forceinline__ void init(int ld, int mn0, int mn_total, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int q = wave * NL + i;
      if (KMAJ) {
        const int row = q * 8 + (lane >> 3), pos = lane & 7;
        const int kc = pos ^ ((row >> 1) & 7);
        int grow = mn0 + row;
        grow = grow < mn_total ? grow : mn_total - 1;
        voff[i] = ((uint32_t)grow * (uint32_t)ld + kc * 8) * 2;
      } else {
        constexpr int CPR = ROWS / 8;  // chunks per k-row
        const int idx = q * 64 + lane, kr = idx / CPR, pos = idx % CPR;
        const int mc = pos ^ kswz<ROWS>(kr);
        int gmn = mn0 + mc * 8;
        gmn = gmn < mn_total ? gmn : mn_total - 8;
        voff[i] = ((uint32_t)kr * (uint32_t)ld + gmn) * 2;
      }
    }
  }
  __device__ __forceinline__ void issue(i32x4 rsrc, bf16_t* tile, uint32_t soff, int wave) const {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int q = wave * NL + i;
      const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)((lds_void_ptr)(tile + q * 512)));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :: "s"(lds_addr), "v"(voff[i]), "s"(rsrc), "s"(soff) : "memory");
    }
  }
};

template <int ROWS, bool KMAJ>
__device__ __forceinline__ bf16x8 read_frag_swz(const bf16_t* tile, int r0, int ks, int lane) {
  if (KMAJ) {
    const int row = r0 + (lane & 31), kc = (ks >> 3) + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(tile + row * 64 + ((kc ^ ((row >> 1) & 7)) << 3));
  } else {
    const int g = lane >> 4, j = lane & 15;
    const int kr = ks + 8 * (g >> 1) + (j >> 2);  // the swizzle is the same for kr and kr + 4
    const int col = r0 + 16 * (g & 1) + 4 * (j & 3);
    const bf16_t* p = tile + kr * ROWS + (col ^ (kswz<ROWS>(kr) << 3));
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * ROWS));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
}

// One output tile (tile_m, tile_n) over the K tiles kt0 .. kt0 + nk - 1: ring prologue, K loop,
// staged epilogue.  All waves of the workgroup call it together; on return the LDS ring holds
// epilogue slabs that other waves may still be reading (barrier before the ring is filled again).
// BK = 32 (both operands [k][rows] only): kt0 and nk count 32-wide K tiles, two 16-wide steps per tile.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KMAJ, bool B_KMAJ, int NSTAGE, int EPI, bool SEG = false, int BK = 64>
__device__ __forceinline__ void dma_tile(const GemmParams& p, bf16_t* smem, int tile_m, int tile_n, int kt0, int nk) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int NW = WAVES_M * WAVES_N, WM = BM / WAVES_M, WN = BN / WAVES_N, TM = WM / 32, TN = WN / 32;
  constexpr int TA = BM * BK, TB = BN * BK, STAGE = TA + TB;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  auto make_rsrc = [](const void* ptr) {  // raw buffer descriptor: base, no stride, 2 GB window
    const uint64_t a = (uint64_t)ptr;
    i32x4 r = {(int)(uint32_t)a, (int)(uint32_t)(a >> 32), 0x7fffffff, 0x00020000};
    return r;
  };
  i32x4 ra = make_rsrc(p.A), rb = make_rsrc(p.B);
  DmaLoader<BM, A_KMAJ, NW, BK> la;
  DmaLoader<BN, B_KMAJ, NW, BK> lb;
  la.init(p.lda, m0, p.M, wave, lane);
  lb.init(p.ldb, n0, p.N, wave, lane);
  const uint32_t stepa = A_KMAJ ? BK * 2 : (uint32_t)BK * p.lda * 2;
  const uint32_t stepb = B_KMAJ ? BK * 2 : (uint32_t)BK * p.ldb * 2;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 fa[2][TM], fb[2][TN];
  // One 16-wide K step: the MFMAs on fragment set c, interleaved in a fixed order with the LDS
  // reads that fill set c^1 from (src_a, src_b) at K offset ks.
  auto step = [&](int c, const bf16_t* src_a, const bf16_t* src_b, int ks) {
#pragma unroll
    for (int q = 0; q < TM + TN; ++q) {
      if (q < TM) fa[c ^ 1][q] = read_frag_swz<BM, A_KMAJ>(src_a, wm0 + 32 * q, ks, lane);
      else fb[c ^ 1][q - TM] = read_frag_swz<BN, B_KMAJ>(src_b, wn0 + 32 * (q - TM), ks, lane);
      __builtin_amdgcn_sched_barrier(0);
      constexpr int NP = TM + TN, TOT = TM * TN;
#pragma unroll
      for (int idx = (q * TOT) / NP; idx < ((q + 1) * TOT) / NP; ++idx) {
        const int i = idx / TN, j = idx % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c][j], fa[c][i], acc[i][j], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Ring of NSTAGE stages.  Tiles past the end are clamped (fetched again, never used) so that the
  // number of loads in flight is the same at every wait.
  constexpr int LPT = DmaLoader<BM, A_KMAJ, NW, BK>::NL + DmaLoader<BN, B_KMAJ, NW, BK>::NL;  // loads per tile per wave
  constexpr int INFL = (NSTAGE - 2) * LPT;  // loads that may stay in flight at a wait
  static_assert(INFL < 64, "vmcnt is a 6-bit field");
  constexpr int WAIT_TILE = (INFL & 15) | ((INFL >> 4) << 14) | (7 << 4) | (15 << 8);  // s_waitcnt vmcnt(INFL)
  auto tile_k = [&](int t) { return kt0 + (t < nk ? t : nk - 1); };
  // Requests K tile t of this call into a stage.  Segmented: tile kt0 + t of the concatenated axis
  // is tile `local` of piece `seg`; the two are stepped along with the requests (which come in
  // ascending t), so no division sits in the loop.
  int seg = 0, local = 0;
  const int seg_tiles = SEG ? p.seg_tiles * (64 / BK) : 0;  // K tiles of this depth per piece
  if (SEG) {
    seg = kt0 / seg_tiles;
    local = kt0 - seg * seg_tiles;
    ra = make_rsrc(p.Aseg[seg]);
    rb = make_rsrc(p.Bseg[seg]);
  }
  auto request = [&](int t, int stage) {
    const int kt = SEG ? local : tile_k(t);
    la.issue(ra, smem + stage * STAGE, kt * stepa, wave);
    lb.issue(rb, smem + stage * STAGE + TA, kt * stepb, wave);
    if (SEG && t + 1 < nk) {  // past the end the last tile is requested again
      if (++local == seg_tiles) {
        local = 0;
        ++seg;
        ra = make_rsrc(p.Aseg[seg]);
        rb = make_rsrc(p.Bseg[seg]);
      }
    }
  };
#pragma unroll
  for (int t = 0; t < NSTAGE - 1; ++t) request(t, t);
  __builtin_amdgcn_s_waitcnt(WAIT_TILE);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) fa[0][i] = read_frag_swz<BM, A_KMAJ>(smem, wm0 + 32 * i, 0, lane);
#pragma unroll
  for (int j = 0; j < TN; ++j) fb[0][j] = read_frag_swz<BN, B_KMAJ>(smem + TA, wn0 + 32 * j, 0, lane);
  int cur = 0;
  for (int kt = 0; kt < nk; ++kt) {
    const bf16_t* cur_a = smem + cur * STAGE;
    const bf16_t* cur_b = cur_a + TA;
    const int nxt = cur + 1 == NSTAGE ? 0 : cur + 1;
    const int fill = cur == 0 ? NSTAGE - 1 : cur - 1;  // all its readers passed the last barrier
    request(kt + NSTAGE - 1, fill);
    step(0, cur_a, cur_b, 16);
    if constexpr (BK == 64) {
      step(1, cur_a, cur_b, 32);
      step(0, cur_a, cur_b, 48);
    }
    // Tile kt+1 must have landed (younger tiles may still be in flight).  Every fragment of tile
    // kt is in registers, so after this barrier its stage may be refilled.
    __builtin_amdgcn_s_waitcnt(WAIT_TILE);
    __syncthreads();
    step(1, smem + nxt * STAGE, smem + nxt * STAGE + TA, 0);  // after the last tile: a clamped tile, unused
    cur = nxt;
  }
  // vmcnt(0): drain the clamped tail loads; after the barrier no wave reads or fills a stage any
  // more and the ring is reused for the epilogue slabs.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  constexpr int JN = TN == 5 ? 4 : TN;  // widest column group of the staged epilogue
  static_assert(NW * 32 * (32 * JN + 4) * 4 <= NSTAGE * STAGE * 2, "epilogue slabs must fit in the stage ring");
  float* slab = reinterpret_cast<float*>(smem) + wave * (32 * (32 * JN + 4));
  epilogue_staged<TM, TN, EPI, 0, JN>(p, acc, slab, m0 + wm0, n0 + wn0, lane);
  if constexpr (TN == 5) epilogue_staged<TM, TN, EPI, 4, 1>(p, acc, slab, m0 + wm0, n0 + wn0, lane);
#endif
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KMAJ, bool B_KMAJ, int NSTAGE, int EPI, bool SEG = false, int BK = 64>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_bf16_dma_kernel(GemmParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  int tile_m, tile_n;
  tile_of_block(p, tile_m, tile_n);
  const int nk = p.k_tiles_per_split * (64 / BK);
  dma_tile<BM, BN, WAVES_M, WAVES_N, A_KMAJ, B_KMAJ, NSTAGE, EPI, SEG, BK>(p, smem, tile_m, tile_n, (int)blockIdx.y * nk, nk);
#endif
}

// Weight-gradient products (fp32 C += A^T B) with several rounds of tiles per compute unit: one
// persistent workgroup per unit walks its tiles.  The read-modify-write of C runs at HBM speed and
// the K loop at matrix-core speed, and a workgroup cannot do both at once; if all workgroups start
// together they stay in step, every K loop finds the memory idle and every epilogue finds it
// saturated.  So the workgroups are put out of phase, without idling anyone: group g of G (by
// workgroup id) starts its first tile at K tile g/G of the way through, and comes back for that
// tile's first K tiles after its last tile.  Both parts are added into C by the same workgroup, in
// that order, so the result depends on the launch shape alone.
template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE, int GROUPS, bool SEG = false, int BK = 64>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_bf16_wgrad_persistent_kernel(GemmParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  const int ntiles = p.tiles_m * p.tiles_n, G = gridDim.x, b = blockIdx.x;
  const int nk = p.k_tiles_per_split * (64 / BK);  // all of K, in tiles of this depth
  const int group = (b >> 3) % GROUPS;  // neighbours on one XCD fall into different groups
  const int head = (nk * group) / GROUPS;  // K tiles of the first tile left for the end
  bool first = true;
  int tm0 = 0, tn0 = 0;
  for (int pid = b; pid < ntiles; pid += G) {
    int tile_m, tile_n;
    tile_of_pid(p, pid, tile_m, tile_n);
    if (first) {
      tm0 = tile_m;
      tn0 = tile_n;
      dma_tile<BM, BN, WAVES_M, WAVES_N, false, false, NSTAGE, PMC_EPI_ACCUM_F32, SEG, BK>(p, smem, tile_m, tile_n, head, nk - head);
      first = false;
    } else {
      dma_tile<BM, BN, WAVES_M, WAVES_N, false, false, NSTAGE, PMC_EPI_ACCUM_F32, SEG, BK>(p, smem, tile_m, tile_n, 0, nk);
    }
    __syncthreads();
  }
  if (!first && head > 0)
    dma_tile<BM, BN, WAVES_M, WAVES_N, false, false, NSTAGE, PMC_EPI_ACCUM_F32, SEG, BK>(p, smem, tm0, tn0, 0, head);
#endif
}

// Weight-gradient products, two workgroups per compute unit: 256x128 tiles, four waves of 128x64
// (the same wave tile as the kernels above, so the same LDS traffic per matrix instruction), a ring of
// three 32-deep stages (72 KB).  Two such workgroups fit a compute unit (144 KB of LDS, two waves per
// SIMD), each with its own barriers: while one adds its finished tile into C at memory speed, the other
// runs its K loop, without any arrangement between them, and the two waves of a SIMD no longer wait at
// the same barrier.  Both operands of a weight gradient are stored [k][rows], so a 32-deep tile still
// reads whole 256- and 512-byte rows.
template <bool SEG>
__global__ __launch_bounds__(256, 2) void gemm_bf16_wgrad_pair_kernel(GemmParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  int tile_m, tile_n;
  tile_of_block(p, tile_m, tile_n);
  dma_tile<256, 128, 2, 2, false, false, 3, PMC_EPI_ACCUM_F32, SEG, 32>(p, smem, tile_m, tile_n, 0, 2 * p.k_tiles_per_split);
#endif
}

// ---------------------------------------------------------------------------------------------
// General path.
template <int BM, int BN, int BK, int WM, int WN, bool A_KMAJ, bool B_KMAJ, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_kernel(GemmParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int WAVES_N = BN / WN;
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int TM = WM / 32, TN = WN / 32;
  using TileA = Tile<BM, BK, A_KMAJ>;
  using TileB = Tile<BN, BK, B_KMAJ>;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  constexpr int kStage = TileA::elems + TileB::elems;  // one buffer: A tile then B tile

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  int tile_m, tile_n;
  tile_of_block(p, tile_m, tile_n);
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

  epilogue<TM, TN, EPI>(p, acc, m0 + wm0, n0 + wn0, lane);
#endif
}

template <int BM, int BN, int BK, int WM, int WN, bool A_KMAJ, bool B_KMAJ, int EPI>
int launch(hipStream_t st, GemmParams p) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr size_t lds = 2 * sizeof(bf16_t) * (Tile<BM, BK, A_KMAJ>::elems + Tile<BN, BK, B_KMAJ>::elems);
  static_assert(lds <= 160 * 1024, "tile does not fit the 160 KB LDS");
  auto kern = gemm_bf16_kernel<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, EPI>;
  static std::atomic<bool> configured{false};  // per instantiation
  if (int rc = reserve_lds(kern, lds, configured, "gemm_bf16")) return rc;
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  p.group_m = 8;
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
    case PMC_EPI_BIAS_GELU_GRAD: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_BIAS_GELU_GRAD>(st, p);
    case PMC_EPI_MUL: return launch<BM, BN, BK, WM, WN, A_KMAJ, B_KMAJ, PMC_EPI_MUL>(st, p);
  }
  return fail(PMC_ERR_INVALID, "gemm_bf16: unknown epilogue %d", epi);
}

template <bool A_KMAJ, bool B_KMAJ>
int launch_tile(hipStream_t st, const GemmParams& p, int epi) {
  return launch_epi<128, 128, 64, 64, 64, A_KMAJ, B_KMAJ>(st, p, epi);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KMAJ, bool B_KMAJ, int NSTAGE, int EPI, bool SEG = false, int BK = 64>
int launch_dma(hipStream_t st, GemmParams p) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr size_t lds = (size_t)NSTAGE * (BM + BN) * BK * sizeof(bf16_t);
  static_assert(lds <= 160 * 1024, "stages do not fit the 160 KB LDS");
  auto kern = gemm_bf16_dma_kernel<BM, BN, WAVES_M, WAVES_N, A_KMAJ, B_KMAJ, NSTAGE, EPI, SEG, BK>;
  static std::atomic<bool> configured{false};  // per instantiation
  if (int rc = reserve_lds(kern, lds, configured, "gemm_bf16")) return rc;
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  {
    const int forced = tuning(kTuneGemmGroup);
    p.group_m = forced > 0 ? forced : (BM >= 256 ? 4 : 8);
  }
  const int splits = (p.K / 64) / p.k_tiles_per_split;
  kern<<<dim3(p.tiles_m * p.tiles_n, splits), dim3(NT), lds, st>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "gemm_bf16 launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

// Tile shape for the fast path.  Tiles are dealt over the 256 compute units, so the time is
// (tiles per unit, rounded up) x (work of a tile) / (throughput of that shape on a busy unit); the
// largest tile wins once there are enough tiles, smaller ones when units would otherwise idle.
//   0: 256x256, 8 waves, 2 stages    1: 256x128, 8 waves, 3 stages    2: 128x128, 4 waves, 2 stages
//   3: 64x128, 4 waves, 3 stages (skinny outputs: twice the tiles of shape 2)
//   4: 256x320, 8 waves, 2 stages (N a multiple of 320 whose 256-wide tiles would leave a ragged last
//      round, e.g. 4096 x 5120 = exactly 256 tiles)
// The gemm_tile tuning switch (0..4) forces a shape (for tests and tuning).
int pick_tile(int M, int N, bool wide_ok) {
  if (const int f = tuning(kTuneGemmTile); f >= 0) return (f == 4 && !wide_ok) ? 0 : f;
  const int bm[5] = {256, 256, 128, 64, 256}, bn[5] = {256, 128, 128, 128, 320};
  const double rate[5] = {1.0, 0.95, 0.75, 0.6, 1.02};  // on a tie in rounds x area the 320-wide tile wins (fewer rounds)
  int best = 0;
  double best_t = 1e300;
  for (int c = 0; c < (wide_ok ? 5 : 4); ++c) {
    const long n = (long)((M + bm[c] - 1) / bm[c]) * ((N + bn[c] - 1) / bn[c]);
    const double t = (double)((n + 255) / 256) * bm[c] * bn[c] / rate[c];
    if (t < best_t) {
      best_t = t;
      best = c;
    }
  }
  return best;
}

template <bool A_KMAJ, bool B_KMAJ, int EPI, bool SEG = false>
int launch_dma_tile(hipStream_t st, const GemmParams& p) {
  // the 320-wide tile holds 10 accumulator tiles per wave; with the fp32 read-modify-write epilogue on
  // top it would spill registers, so weight-gradient products do not use it
  constexpr bool kWideOk = EPI != PMC_EPI_ACCUM_F32;
  switch (pick_tile(p.M, p.N, kWideOk)) {
    case 0:
      // both operands stored [k][rows] (weight gradients): four 32-deep stages instead of two 64-deep ones, see
      // launch_wgrad_persistent
      if constexpr (!A_KMAJ && !B_KMAJ) return launch_dma<256, 256, 2, 4, A_KMAJ, B_KMAJ, 4, EPI, SEG, 32>(st, p);
      else return launch_dma<256, 256, 2, 4, A_KMAJ, B_KMAJ, 2, EPI, SEG>(st, p);
    case 1: return launch_dma<256, 128, 4, 2, A_KMAJ, B_KMAJ, 3, EPI, SEG>(st, p);
    case 4:
      if constexpr (kWideOk) return launch_dma<256, 320, 4, 2, A_KMAJ, B_KMAJ, 2, EPI, SEG>(st, p);
      else return launch_dma<256, 256, 2, 4, A_KMAJ, B_KMAJ, 2, EPI, SEG>(st, p);
    case 3:  // the [64 k][rows] swizzle needs 128 rows: a 64-row A tile only when A is contraction-contiguous
      if constexpr (A_KMAJ) return launch_dma<64, 128, 1, 4, A_KMAJ, B_KMAJ, 3, EPI, SEG>(st, p);
      else return launch_dma<128, 128, 2, 2, A_KMAJ, B_KMAJ, 2, EPI, SEG>(st, p);
    default: return launch_dma<128, 128, 2, 2, A_KMAJ, B_KMAJ, 2, EPI, SEG>(st, p);
  }
}

// Compute units of the current device, asked once (0 if the query fails).
int compute_units() {
  static std::atomic<int> units{0};
  int u = units.load(std::memory_order_relaxed);
  if (u > 0) return u;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
  units.store(prop.multiProcessorCount, std::memory_order_relaxed);
  return prop.multiProcessorCount;
}

// Persistent, phase-shifted weight-gradient kernel: when every compute unit gets at least two
// 256x256 tiles.  The gemm_wgrad tuning switch (0|1) forces the choice (tests, tuning).
bool use_wgrad_persistent(const GemmParams& p) {
  if (p.K < 4 * 64) return false;
  if (const int f = tuning(kTuneGemmWgrad); f >= 0) return f == 1;
  if (tuning(kTuneGemmTile) >= 0) return false;
  return (long)((p.M + 255) / 256) * ((p.N + 255) / 256) >= 2 * 256;
}

template <bool SEG>
int launch_wgrad_persistent(hipStream_t st, GemmParams p) {
  // measured: 2 phases give the most (1: -6 % W-pass time, 2: -8 %, 4 and 8: -7 %).  The ring is four 32-deep
  // stages rather than two 64-deep ones: the same LDS, but a tile is requested three steps (1.5 times as
  // far) ahead of its use, which the weight gradient's operand panels, the least shared in L2 of all products,
  // need most; both operands are stored [k][rows], so a 32-deep tile still reads whole rows.  Measured on
  // whole steps: W pass -3 % at 4096 tokens, -5 % at 2048.
  constexpr int NSTAGE = 4, GROUPS = 2, BK = 32;
  constexpr size_t lds = (size_t)NSTAGE * (256 + 256) * BK * sizeof(bf16_t);
  auto kern = gemm_bf16_wgrad_persistent_kernel<256, 256, 2, 4, NSTAGE, GROUPS, SEG, BK>;
  static std::atomic<bool> configured{false};
  if (int rc = reserve_lds(kern, lds, configured, "gemm_bf16")) return rc;
  const int units = compute_units();
  if (units <= 0) return fail(PMC_ERR_HIP, "gemm_bf16: cannot query the device");
  p.tiles_m = (p.M + 255) / 256;
  p.tiles_n = (p.N + 255) / 256;
  p.group_m = 8;
  const int ntiles = p.tiles_m * p.tiles_n;
  int grid = ntiles < units ? ntiles : units;
  if (grid >= 8) grid &= ~7;  // whole rounds over the 8 XCDs keep a workgroup's tiles on one XCD
  kern<<<dim3(grid), dim3(512), lds, st>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "gemm_bf16 weight-gradient launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

// The two-workgroup kernel pays 1.5x the operand traffic of 256x256 tiles and a barrier every 16 matrix
// instructions; it wins where the K loop is short, so that a tile's ring fill and read-modify-write
// epilogue weigh as much as its K loop (measured on whole steps: -5 % of the W pass at 1024 tokens,
// +6 % at 2048, +26 % at 4096).  Taking it for some of a layer's products only (those with 256 tiles
// or more) was slower than taking it for none, so the bar on the tile count is low.  gemm_wgrad = 2 forces it.
bool use_wgrad_pair(const GemmParams& p) {
  if (const int f = tuning(kTuneGemmWgrad); f >= 0) return f == 2;
  if (tuning(kTuneGemmTile) >= 0) return false;
  return p.K <= 1024 && (long)((p.M + 255) / 256) * ((p.N + 127) / 128) >= 64;
}

template <bool SEG>
int launch_wgrad_pair(hipStream_t st, GemmParams p) {
  constexpr size_t lds = (size_t)3 * (256 + 128) * 32 * sizeof(bf16_t);
  auto kern = gemm_bf16_wgrad_pair_kernel<SEG>;
  static std::atomic<bool> configured{false};
  if (int rc = reserve_lds(kern, lds, configured, "gemm_bf16")) return rc;
  p.tiles_m = (p.M + 255) / 256;
  p.tiles_n = (p.N + 127) / 128;
  {
    const int forced = tuning(kTuneGemmGroup);
    p.group_m = forced > 0 ? forced : 4;
  }
  kern<<<dim3(p.tiles_m * p.tiles_n), dim3(256), lds, st>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "gemm_bf16 weight-gradient launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

// Split K: when even 128x128 tiles leave most compute units idle (skinny products such as the
// [tokens, hidden] outputs at short sequence length), K is cut into `splits` ranges, each range
// writes an fp32 partial product to the workspace and a second kernel adds them and applies the
// epilogue.  Returns 1 when splitting does not pay or does not fit.
int pick_splits(int M, int N, int K, size_t ws_bytes) {
  if (tuning(kTuneGemmTile) >= 0) return 1;
  const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
  if (tiles >= 192) return 1;
  // up to K = 6144 the 64x128 tiles (no partials, no second kernel) are faster once there are
  // enough of them (measured at M = 1024, N = 2048: 15 / 38 us against 27 / 41 us at K = 2048 / 6144)
  if (K < 8192 && (long)((M + 63) / 64) * ((N + 127) / 128) >= 192) return 1;
  const int nkt = K / 64;
  int best = 1;
  for (int s : {2, 4, 8}) {
    if (nkt % s || nkt / s < 4) continue;                          // whole tiles, at least 256 of K per split
    if ((size_t)s * M * N * sizeof(float) > ws_bytes) break;
    best = s;
    if (tiles * s >= 384) break;
  }
  return best;
}

template <bool A_KMAJ, bool B_KMAJ>
int launch_partial(hipStream_t st, GemmParams p, void* ws, int splits) {
  p.C = ws;
  p.k_tiles_per_split = (p.K / 64) / splits;
  return launch_dma<128, 128, 2, 2, A_KMAJ, B_KMAJ, 2, kEpiPartial>(st, p);
}

template <int EPI>
int launch_reduce_epi(hipStream_t st, const GemmParams& p, const float* ws, int splits) {
  const size_t quads = (size_t)p.M * p.N / 4;
  splitk_reduce_kernel<EPI><<<dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st>>>(p, ws, splits);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "gemm_bf16 split-K reduce launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

int launch_reduce(hipStream_t st, const GemmParams& p, const float* ws, int splits, int epi) {
  switch (epi) {
    case PMC_EPI_NONE: return launch_reduce_epi<PMC_EPI_NONE>(st, p, ws, splits);
    case PMC_EPI_BIAS: return launch_reduce_epi<PMC_EPI_BIAS>(st, p, ws, splits);
    case PMC_EPI_BIAS_RESID: return launch_reduce_epi<PMC_EPI_BIAS_RESID>(st, p, ws, splits);
    case PMC_EPI_BIAS_GELU: return launch_reduce_epi<PMC_EPI_BIAS_GELU>(st, p, ws, splits);
    case PMC_EPI_DGELU: return launch_reduce_epi<PMC_EPI_DGELU>(st, p, ws, splits);
    case PMC_EPI_ACCUM_F32: return launch_reduce_epi<PMC_EPI_ACCUM_F32>(st, p, ws, splits);
    case PMC_EPI_BIAS_GELU_GRAD: return launch_reduce_epi<PMC_EPI_BIAS_GELU_GRAD>(st, p, ws, splits);
    case PMC_EPI_MUL: return launch_reduce_epi<PMC_EPI_MUL>(st, p, ws, splits);
  }
  return fail(PMC_ERR_INVALID, "gemm_bf16: unknown epilogue %d", epi);
}

// The layout/epilogue combinations the passes use (and the plain product of each layout) have a
// fast-path instantiation; returns -100 if this combination has none.
constexpr int kNoFastPath = -100;
int launch_fast(hipStream_t st, const GemmParams& p, bool a_kmaj, bool b_kmaj, int epi) {
  if (a_kmaj && !b_kmaj) {  // F: Y = X . W
    switch (epi) {
      case PMC_EPI_NONE: return launch_dma_tile<true, false, PMC_EPI_NONE>(st, p);
      case PMC_EPI_BIAS: return launch_dma_tile<true, false, PMC_EPI_BIAS>(st, p);
      case PMC_EPI_BIAS_RESID: return launch_dma_tile<true, false, PMC_EPI_BIAS_RESID>(st, p);
      case PMC_EPI_BIAS_GELU: return launch_dma_tile<true, false, PMC_EPI_BIAS_GELU>(st, p);
      case PMC_EPI_BIAS_GELU_GRAD: return launch_dma_tile<true, false, PMC_EPI_BIAS_GELU_GRAD>(st, p);
    }
  } else if (a_kmaj && b_kmaj) {  // B: dX = dY . W^T
    switch (epi) {
      case PMC_EPI_NONE: return launch_dma_tile<true, true, PMC_EPI_NONE>(st, p);
      case PMC_EPI_DGELU: return launch_dma_tile<true, true, PMC_EPI_DGELU>(st, p);
      case PMC_EPI_MUL: return launch_dma_tile<true, true, PMC_EPI_MUL>(st, p);
    }
  } else if (!a_kmaj && !b_kmaj) {  // W: dW += X^T . dY
    switch (epi) {
      case PMC_EPI_NONE: return launch_dma_tile<false, false, PMC_EPI_NONE>(st, p);
      case PMC_EPI_ACCUM_F32: return launch_dma_tile<false, false, PMC_EPI_ACCUM_F32>(st, p);
    }
  }
  return kNoFastPath;
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
  p.group_m = 8;
  p.k_tiles_per_split = 0;
  p.nseg = p.seg_tiles = 0;
  for (int i = 0; i < kMaxSegments; ++i) p.Aseg[i] = p.Bseg[i] = nullptr;
  const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
  // Fast path: K in whole 64-wide tiles, operands inside the 2 GB window of a buffer descriptor.
  const size_t a_bytes = (size_t)(a.trans_a ? a.K : a.M) * a.lda * 2, b_bytes = (size_t)(a.trans_b ? a.N : a.K) * a.ldb * 2;
  if (a.K % 64 == 0 && a_bytes < 0x7fffffffull && b_bytes < 0x7fffffffull) {
    p.k_tiles_per_split = a.K / 64;
    const int splits = (a.ws && !(a_kmaj == false && b_kmaj == true)) ? pick_splits(a.M, a.N, a.K, a.ws_bytes) : 1;
    if (splits > 1) {
      int rc = a_kmaj ? (b_kmaj ? launch_partial<true, true>(st, p, a.ws, splits) : launch_partial<true, false>(st, p, a.ws, splits))
                      : launch_partial<false, false>(st, p, a.ws, splits);
      if (rc != PMC_OK) return rc;
      return launch_reduce(st, p, (const float*)a.ws, splits, a.epilogue);
    }
    if (!a_kmaj && !b_kmaj && a.epilogue == PMC_EPI_ACCUM_F32 && use_wgrad_pair(p)) return launch_wgrad_pair<false>(st, p);
    if (!a_kmaj && !b_kmaj && a.epilogue == PMC_EPI_ACCUM_F32 && use_wgrad_persistent(p)) return launch_wgrad_persistent<false>(st, p);
    const int rc = launch_fast(st, p, a_kmaj, b_kmaj, a.epilogue);
    if (rc != kNoFastPath) return rc;
  }
  if (a_kmaj && b_kmaj) return launch_tile<true, true>(st, p, a.epilogue);
  if (a_kmaj && !b_kmaj) return launch_tile<true, false>(st, p, a.epilogue);
  if (!a_kmaj && b_kmaj) return launch_tile<false, true>(st, p, a.epilogue);
  return launch_tile<false, false>(st, p, a.epilogue);
}

// C[M,N] (fp32) += sum over pieces i of A_i^T . B_i, A_i stored [K,M], B_i stored [K,N]: one product
// whose contraction runs through the pieces one after the other, one read-modify-write of C.
int gemm_bf16_grouped_wgrad(hipStream_t st, const GroupedWgradArgs& a) {
  if (a.count < 1 || a.count > kMaxSegments) return fail(PMC_ERR_INVALID, "grouped weight gradient: %d pieces (1..%d)", a.count, kMaxSegments);
  if (a.M % 8 || a.N % 8 || a.K % 64) return fail(PMC_ERR_INVALID, "grouped weight gradient: M=%d N=%d must be multiples of 8, K=%d of 64", a.M, a.N, a.K);
  if (a.lda % 8 || a.ldb % 8 || a.ldc % 4 || a.lda < a.M || a.ldb < a.N || a.ldc < a.N)
    return fail(PMC_ERR_INVALID, "grouped weight gradient: bad pitches (lda=%d ldb=%d ldc=%d)", a.lda, a.ldb, a.ldc);
  if ((size_t)a.K * a.lda * 2 >= 0x7fffffffull || (size_t)a.K * a.ldb * 2 >= 0x7fffffffull)
    return fail(PMC_ERR_INVALID, "grouped weight gradient: a piece exceeds the 2 GB window of a buffer descriptor");
  if (!aligned(a.C, 16)) return fail(PMC_ERR_INVALID, "grouped weight gradient: C must be 16-byte aligned");
  GemmParams p;
  p.A = (const bf16_t*)a.A[0]; p.B = (const bf16_t*)a.B[0]; p.C = a.C;
  p.bias = p.resid = nullptr; p.aux = nullptr;
  p.M = a.M; p.N = a.N; p.K = a.K * a.count; p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc;
  p.tiles_m = p.tiles_n = 0;
  p.group_m = 8;
  p.k_tiles_per_split = p.K / 64;
  p.nseg = a.count;
  p.seg_tiles = a.K / 64;
  for (int i = 0; i < kMaxSegments; ++i) {
    const int j = i < a.count ? i : a.count - 1;
    if (!a.A[j] || !a.B[j] || !aligned(a.A[j], 16) || !aligned(a.B[j], 16))
      return fail(PMC_ERR_INVALID, "grouped weight gradient: piece %d is NULL or not 16-byte aligned", j);
    p.Aseg[i] = (const bf16_t*)a.A[j];
    p.Bseg[i] = (const bf16_t*)a.B[j];
  }
  if (use_wgrad_pair(p)) return launch_wgrad_pair<true>(st, p);
  if (use_wgrad_persistent(p)) return launch_wgrad_persistent<true>(st, p);
  return launch_dma_tile<false, false, PMC_EPI_ACCUM_F32, true>(st, p);
}

size_t gemm_scratch_bytes(int dtype, int M, int N, int K) {
  if (dtype != PMC_BF16 || K % 64 || M <= 0 || N <= 0) return 0;
  const int splits = pick_splits(M, N, K, (size_t)-1);
  return splits > 1 ? (size_t)splits * M * N * sizeof(float) : 0;
}

}  // namespace k
}  // namespace pmc
