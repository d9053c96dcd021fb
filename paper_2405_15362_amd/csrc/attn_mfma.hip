// Fused flash-style attention for bf16 storage on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16), packed qkv [batch*seq, 3h].  The tiles are 64 or 128 columns wide; a head
// size that is another multiple of 8 runs in the next wider tile with the remaining columns at zero.
//
// Forward: a workgroup owns a block of queries of one head and streams blocks of K and V through
// LDS (double buffered); its waves form a grid over (32-query group, key group).  Scores are
// produced transposed, S^T[key][query], so every lane owns ONE query column: the online-softmax
// max/sum over keys are in-lane reductions plus one exchange between the two half-waves, and the
// probabilities already sit in the register layout of the B operand of the second product
// O^T = V^T . P^T.  V^T is never formed in memory: the V tile stays [key][dh] in LDS and is read
// with the transposing LDS load.  Saves O and the log-sum-exp.
//
// Backward is two kernels, each output element having one writer and a fixed summation order
// (results are reproducible run to run):
//   dQ   per query block, streaming K/V blocks: recomputes P from the saved log-sum-exp,
//        dS = P * (dO.V^T - delta), dQ^T += K^T . dS^T; also emits delta = rowsum(dO * O).
//   dKdV per key block, streaming Q/dO blocks: dV^T += dO^T . P, dK^T += Q^T . dS, written
//        in place over K and V (a key block is read only by the workgroup that owns it).
// The launch shapes are chosen by the number of (128-row block, head) pairs: few pairs get small
// row blocks and more waves per block so that all compute units have work.
#include <cstdlib>

#include "dev_common.h"
#include "kernels.h"

namespace pmc {
namespace k {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSlack = 8.0f;  // forward: how far (in log2 units) a score may exceed the softmax reference

typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
typedef short s16x8 __attribute__((ext_vector_type(8)));

// LDS tiles are [rows][DH] bf16 without padding, filled by direct-to-LDS loads (one wave instruction
// writes 1 KB, lane l the bytes 16 l .. 16 l + 15 of it) and XOR-swizzled in 16-byte chunks: chunk c
// of row r sits at position c ^ swz(r).  swz is chosen so that both read patterns are free of bank
// conflicts: 16 consecutive rows at one chunk fall into 16 different 16-byte bank groups (operand
// fragments along the rows), and the four rows a transposing read touches fall into the four 64-byte
// quarters of the banks.
template <int DH>
__device__ __forceinline__ int swz(int row) {
  return DH == 128 ? (((row & 3) << 2) | ((row >> 2) & 3))           // 16 chunks per 256-byte row
                   : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));   // 8 chunks per 128-byte row, two rows per bank pass
}

// Fragment with the contraction index contiguous in the LDS row: lane l gets row row0 + l%32,
// contraction indices k0 + 8*(l/32) .. +7.
template <int DH>
__device__ __forceinline__ bf16x8 frag_rows(const bf16_t* tile, int row0, int k0, int lane) {
  const int row = row0 + (lane & 31), c = (k0 >> 3) + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(tile + row * DH + ((c ^ swz<DH>(row)) << 3));
}

// Fragment of the TRANSPOSE of an LDS tile: lane l gets tile column col0 + l%32 and, as its 8
// contraction entries, tile rows  krow0 + 4*(l/32) + {0,1,2,3}  and  krow0 + 8 + 4*(l/32) + {0,1,2,3}.
// That row order is exactly the one in which a lane holds a 32x32 accumulator tile's registers
// 8t .. 8t+7 (rows 8*(r/4) + 4*(l/32) + r%4), so accumulators can be fed back as the other operand.
template <int DH>
__device__ __forceinline__ bf16x8 frag_cols(const bf16_t* tile, int col0, int krow0, int lane) {
  const int g = lane >> 4, j = lane & 15;
  const int row = krow0 + 4 * (g >> 1) + (j >> 2), col = col0 + 16 * (g & 1) + 4 * (j & 3);
  const int c = col >> 3, within = col & 7;
  const bf16_t* p = tile + row * DH + ((c ^ swz<DH>(row)) << 3) + within;
  const bf16_t* q = tile + (row + 8) * DH + ((c ^ swz<DH>(row + 8)) << 3) + within;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(q));
  const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// Registers 8t .. 8t+7 of an accumulator tile as a bf16 operand fragment.
__device__ __forceinline__ bf16x8 acc_to_frag(const f32x16& a, int t) {
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (__bf16)a[8 * t + e];
  return v;
}

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// Raw buffer descriptor with a 2 GB window at ptr (every offset used stays below that: checked on the host).
__device__ __forceinline__ i32x4 make_rsrc(const void* ptr) {
  const uint64_t a = (uint64_t)ptr;
  i32x4 r = {(int)(uint32_t)a, (int)(uint32_t)(a >> 32), 0x7fffffff, 0x00020000};
  return r;
}

// Cooperative direct-to-LDS copy of a [ROWS][DH] block of rows (row pitch ld elements in global
// memory) by the NT threads of the workgroup: the data never passes through registers.  Rows past
// the last one are clamped to it, so every access stays inside the tensor; what those rows
// contribute is masked by the caller.  The loads are inline assembly: the caller waits for them
// with s_waitcnt vmcnt(0) before the barrier that publishes the tile.
template <int ROWS, int DH, int NT>
struct BlockDma {
  static constexpr int CPR = DH / 8;                 // chunks per row
  static constexpr int RPI = 64 / CPR;               // rows per wave instruction
  static constexpr int NI = ROWS / RPI;              // wave instructions per block
  static constexpr int NW = NT / 64;
  static constexpr int PER = (NI + NW - 1) / NW;     // per wave (the last waves idle if NI % NW)
  static_assert(ROWS % RPI == 0, "block must be whole wave instructions");
  static constexpr uint32_t kSkip = 0xffffffffu;
  int row_in_block[PER];
  uint32_t col_bytes[PER];
  // dh: columns a row really has (a multiple of 8, at most DH).  Lanes whose chunk lies past them
  // load nothing; their LDS positions keep the zeros the kernel wrote there once.
  __device__ __forceinline__ void init(int wave, int lane, int dh = DH) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = wave + i * NW, row = q * RPI + lane / CPR, pos = lane % CPR;
      const int chunk = pos ^ swz<DH>(row);
      row_in_block[i] = row;
      col_bytes[i] = 8 * chunk < dh ? (uint32_t)(chunk << 4) : kSkip;
    }
  }
  // row0: first row of the block; last_row: the last valid row; ld_bytes: row pitch in bytes
  template <bool PAD = false>
  __device__ __forceinline__ void issue(i32x4 rsrc, bf16_t* tile, uint32_t ld_bytes, int row0, int last_row, int wave) const {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = wave + i * NW;
      if (NI % NW != 0 && q >= NI) break;
      const uint32_t voff = (uint32_t)min(row0 + row_in_block[i], last_row) * ld_bytes + col_bytes[i];
      const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)((lds_void_ptr)(tile + q * 512)));
      if (!PAD || col_bytes[i] != kSkip)  // a lane writes its own 16 bytes of the instruction's 1 KB whoever else is active
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :: "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
    }
  }
};

constexpr int kWaitAllLoads = 0x0F70;  // s_waitcnt vmcnt(0)

__device__ __forceinline__ void zero(f32x16& a) {
#pragma unroll
  for (int r = 0; r < 16; ++r) a[r] = 0.f;
}

// Writes an accumulator tile holding OUT^T[dh][row] (lane = row, registers = dh) times `mul` to
// out[row][col0 + 32*dt + ...] as bf16, four consecutive columns per store; only the first `cols`
// of the tile's 32 columns exist (a multiple of 4).
__device__ __forceinline__ void store_tile_t(bf16_t* row_ptr, const f32x16& a, float mul, int lane, int cols = 32) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    u32x2 v = {pack_bf16x2(a[4 * q] * mul, a[4 * q + 1] * mul), pack_bf16x2(a[4 * q + 2] * mul, a[4 * q + 3] * mul)};
    if (8 * q + 4 * (lane >> 5) < cols) *reinterpret_cast<u32x2*>(row_ptr + 8 * q + 4 * (lane >> 5)) = v;
  }
}

// Eight consecutive elements of a row from global memory, zeros if they lie past the row's dh columns.
__device__ __forceinline__ bf16x8 load_frag(const bf16_t* p, int col, int dh) {
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.f;
  return col < dh ? *reinterpret_cast<const bf16x8*>(p + col) : z;
}

// Head sizes below the tile width: the tiles' columns past dh are zeroed once (the loads skip them).
template <int NT>
__device__ __forceinline__ void zero_tiles(bf16_t* smem, int elems, int tid) {
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (int i = tid * 8; i < elems; i += NT * 8) *reinterpret_cast<u32x4*>(smem + i) = z;
  __syncthreads();
}

// Forward.  The workgroup is a QW x KW grid of waves: wave (qg, kg) owns queries 32 qg .. 32 qg + 31
// of the workgroup's 32 QW queries and, of every streamed block of 32 NKT KW keys, the 32 NKT keys
// starting at 32 NKT kg.
// Each wave runs its own online softmax over the keys it sees; at the end the KW partial results of
// a query group are merged in key-group order through LDS.  Splitting the keys over waves puts two
// waves on every SIMD even when there are few (query block, head) pairs, and shortens the serial
// chain of a long row of key blocks.
// PAD: the head size dh is smaller than the tile width DH (the columns past dh are kept at zero).
template <int DH, int QW, int KW, int NKT, bool PAD>
__global__ __launch_bounds__(QW * KW * 64, QW * KW == 4 ? 2 : 1) void attn_fwd_mfma(int seq, int heads, int dh, int causal, const bf16_t* __restrict__ qkv,
                                                               bf16_t* __restrict__ o, float* __restrict__ lse,
                                                               float scale_log2) {
  constexpr int NT = QW * KW * 64, BQW = 32 * QW, WK = 32 * NKT, BSW = WK * KW;
  constexpr int KT = BSW * DH, VT = BSW * DH;
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];  // [2][K tile | V tile]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hl = lane >> 5;
  const int qg = wave % QW, kg = wave / QW;
  // grid = (heads * batch, query blocks); under a causal mask late query blocks see the most keys,
  // so they are dealt out first and the short ones fill the tail
  const int h = heads * dh, head = blockIdx.x % heads, b = blockIdx.x / heads;
  const int q0 = (causal ? (int)(gridDim.y - 1 - blockIdx.y) : (int)blockIdx.y) * BQW, qw0 = q0 + 32 * qg, qrow = qw0 + (lane & 31);
  const size_t ld = (size_t)3 * h;
  const bf16_t* base = qkv + (size_t)b * seq * ld + (size_t)head * dh;

  bf16x8 qf[DH / 16];
  {
    const bf16_t* qp = base + (size_t)min(qrow, seq - 1) * ld;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) qf[ks] = load_frag(qp, 16 * ks + 8 * hl, PAD ? dh : DH);
  }
  f32x16 oacc[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt) zero(oacc[dt]);
  float m2 = -INFINITY, lsum = 0.f;  // softmax reference (log2 units, scale applied; see below) and sum

  const int kend = causal ? min(seq, q0 + BQW) : seq;
  const int nblk = (kend + BSW - 1) / BSW;
  const i32x4 rk = make_rsrc(base + h), rv = make_rsrc(base + 2 * h);
  const uint32_t ldb = (uint32_t)ld * 2;
  if (PAD) zero_tiles<NT>(smem, 2 * (KT + VT), tid);
  BlockDma<BSW, DH, NT> dma;
  dma.init(wave, lane, PAD ? dh : DH);
  dma.template issue<PAD>(rk, smem, ldb, 0, seq - 1, wave);
  dma.template issue<PAD>(rv, smem + KT, ldb, 0, seq - 1, wave);
  __builtin_amdgcn_s_waitcnt(kWaitAllLoads);
  __syncthreads();
  // The query fragments must have arrived before the loop: left pending, the compiler's wait for
  // them inside the loop would also cover the loads that prefetch the next block.
#pragma unroll
  for (int ks = 0; ks < DH / 16; ++ks) asm volatile("" ::"v"(qf[ks]));
  for (int blk = 0; blk < nblk; ++blk) {
    const int k0 = blk * BSW + WK * kg;  // this wave's 32 NKT keys
    const bf16_t* kt_ = smem + (blk & 1) * (KT + VT);
    const bf16_t* vt_ = kt_ + KT;
    if (blk + 1 < nblk) {  // the other stage: every wave left it at the last barrier
      bf16_t* nxt = smem + ((blk + 1) & 1) * (KT + VT);
      dma.template issue<PAD>(rk, nxt, ldb, (blk + 1) * BSW, seq - 1, wave);
      dma.template issue<PAD>(rv, nxt + KT, ldb, (blk + 1) * BSW, seq - 1, wave);
    }
    if (k0 < seq && (!causal || k0 <= qw0 + 31)) {
      // The K fragments of a 32-key tile are requested together, and those of the next tile each
      // as soon as its register is free, so that the LDS latency is paid once, not per product; the
      // first V fragments are requested before the softmax arithmetic for the same reason.
      f32x16 s[NKT];
      bf16x8 kf[DH / 16];
#pragma unroll
      for (int ks = 0; ks < DH / 16; ++ks) kf[ks] = frag_rows<DH>(kt_, WK * kg, 16 * ks, lane);
      __builtin_amdgcn_sched_barrier(0);  // the compiler would sink the reads to their uses again
#pragma unroll
      for (int kt = 0; kt < NKT; ++kt) {
        zero(s[kt]);
#pragma unroll
        for (int ks = 0; ks < DH / 16; ++ks) {
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], s[kt], 0, 0, 0);
          if (kt + 1 < NKT) kf[ks] = frag_rows<DH>(kt_, WK * kg + 32 * (kt + 1), 16 * ks, lane);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      bf16x8 vf[2][DH / 32];
#pragma unroll
      for (int dt = 0; dt < DH / 32; ++dt) vf[0][dt] = frag_cols<DH>(vt_, 32 * dt, WK * kg, lane);
      __builtin_amdgcn_sched_barrier(0);
      // only blocks that cross the diagonal of this wave's rows or the end of the sequence need masks
      if ((causal && k0 + WK - 1 > qw0) || (k0 + WK > seq)) {
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + 32 * kt + 8 * (r >> 2) + 4 * hl + (r & 3);
            if (key >= seq || (causal && key > qrow)) s[kt][r] = -INFINITY;
          }
      }
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // m2 is the reference the exponentials are taken against, not necessarily the exact running
      // maximum: it moves (and what is summed so far is rescaled) only when some query's maximum
      // has risen by more than kSlack above it, so probabilities stay below 2^kSlack and the
      // quotient o / lsum and lse = m2 + log2(lsum) are the same as with the exact maximum.
      const float m_new = fmaxf(m2, mx * scale_log2);
      if (__any(m_new > m2 + kSlack)) {
        const float alpha = __builtin_amdgcn_exp2f(m2 - ((m_new == -INFINITY) ? 0.f : m_new));
        lsum *= alpha;
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
        m2 = m_new;
      }
      const float m_use = (m2 == -INFINITY) ? 0.f : m2;
      float rowsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][r], scale_log2, -m_use));
          s[kt][r] = p;
          rowsum += p;
        }
      rowsum += __shfl_xor(rowsum, 32, 64);
      lsum += rowsum;
#pragma unroll
      for (int g = 0; g < 2 * NKT; ++g) {  // 16 keys at a time: tile g / 2, half g % 2
        if (g + 1 < 2 * NKT) {
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt) vf[(g + 1) & 1][dt] = frag_cols<DH>(vt_, 32 * dt, WK * kg + 16 * (g + 1), lane);
        }
        const bf16x8 pb = acc_to_frag(s[g >> 1], g & 1);
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[g & 1][dt], pb, oacc[dt], 0, 0, 0);
      }
    }
    __builtin_amdgcn_s_waitcnt(kWaitAllLoads);  // this wave's part of the next block has landed
    __syncthreads();
  }
  if (KW > 1) {
    // Merge the key groups of each query group: groups 1.. park (O, m, l) in LDS (the tiles are no
    // longer read), group 0 folds them in ascending order.  Slot layout: [DH/2 + 2][64 lanes] fp32.
    constexpr int SLOT = (DH / 2 + 2) * 64;
    static_assert((size_t)QW * (KW - 1) * SLOT * 4 <= (size_t)2 * (KT + VT) * 2, "merge slots must fit in the tiles");
    float* slots = reinterpret_cast<float*>(smem);
    if (kg > 0) {
      float* my = slots + ((kg - 1) * QW + qg) * SLOT;
#pragma unroll
      for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) my[(dt * 16 + r) * 64 + lane] = oacc[dt][r];
      my[(DH / 2) * 64 + lane] = m2;
      my[(DH / 2 + 1) * 64 + lane] = lsum;
    }
    __syncthreads();
    if (kg > 0) return;
#pragma unroll 1
    for (int g = 1; g < KW; ++g) {
      const float* other = slots + ((g - 1) * QW + qg) * SLOT;
      const float mo = other[(DH / 2) * 64 + lane], lo = other[(DH / 2 + 1) * 64 + lane];
      const float m_new = fmaxf(m2, mo);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float a = __builtin_amdgcn_exp2f(m2 - m_use), bo = __builtin_amdgcn_exp2f(mo - m_use);
      lsum = lsum * a + lo * bo;
#pragma unroll
      for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = oacc[dt][r] * a + other[(dt * 16 + r) * 64 + lane] * bo;
      m2 = m_new;
    }
  }
  if (qrow < seq) {
    const float inv = 1.0f / lsum;
    bf16_t* orow = o + ((size_t)b * seq + qrow) * h + (size_t)head * dh;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt) store_tile_t(orow + 32 * dt, oacc[dt], inv, lane, PAD ? dh - 32 * dt : 32);
    if (hl == 0) lse[((size_t)b * heads + head) * seq + qrow] = (m2 + log2f(lsum)) * kLn2;
  }
}

// Backward, dQ.  Same wave grid as the forward kernel: wave (qg, kg) owns 32 queries and the 32 NKT
// keys starting at 32 NKT kg of every streamed block; 32-key tiles are taken one at a time
// (S and dP, then dS, then dQ^T += K^T dS^T) to keep the register footprint at two waves per SIMD.
// The KW partial dQ of a query group are added in key-group order through LDS at the end.
template <int DH, int QW, int KW, int NKT, bool PAD>
__global__ __launch_bounds__(QW * KW * 64, QW * KW == 4 ? 2 : 1) void attn_bwd_dq_mfma(
    int seq, int heads, int dh, int causal, const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
    const float* __restrict__ lse, const bf16_t* __restrict__ d_o, bf16_t* __restrict__ dq, float* __restrict__ delta,
    float scale, float scale_log2) {
  constexpr int NT = QW * KW * 64, BQW = 32 * QW, WK = 32 * NKT, BSW = WK * KW;
  constexpr int KT = BSW * DH, VT = BSW * DH;
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hl = lane >> 5;
  const int qg = wave % QW, kg = wave / QW;
  // grid = (heads * batch, query blocks); under a causal mask late query blocks see the most keys,
  // so they are dealt out first and the short ones fill the tail
  const int h = heads * dh, head = blockIdx.x % heads, b = blockIdx.x / heads;
  const int q0 = (causal ? (int)(gridDim.y - 1 - blockIdx.y) : (int)blockIdx.y) * BQW, qw0 = q0 + 32 * qg, qrow = qw0 + (lane & 31);
  const int qclamp = min(qrow, seq - 1);
  const size_t ld = (size_t)3 * h;
  const bf16_t* base = qkv + (size_t)b * seq * ld + (size_t)head * dh;

  bf16x8 qf[DH / 16], dof[DH / 16];
  float dl = 0.f;
  {
    const bf16_t* qp = base + (size_t)qclamp * ld;
    const size_t orow = ((size_t)b * seq + qclamp) * h + (size_t)head * dh;
    const int cols = PAD ? dh : DH;
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
      qf[ks] = load_frag(qp, 16 * ks + 8 * hl, cols);
      dof[ks] = load_frag(d_o + orow, 16 * ks + 8 * hl, cols);
      const bf16x8 of = load_frag(o + orow, 16 * ks + 8 * hl, cols);
#pragma unroll
      for (int e = 0; e < 8; ++e) dl += (float)dof[ks][e] * (float)of[e];
    }
  }
  dl += __shfl_xor(dl, 32, 64);
  const size_t stat = ((size_t)b * heads + head) * seq + qclamp;
  if (kg == 0 && hl == 0 && qrow < seq) delta[stat] = dl;
  const float lse2 = lse[stat] * kLog2e;
  f32x16 acc[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt) zero(acc[dt]);

  const int kend = causal ? min(seq, q0 + BQW) : seq;
  const int nblk = (kend + BSW - 1) / BSW;
  const i32x4 rk = make_rsrc(base + h), rv = make_rsrc(base + 2 * h);
  const uint32_t ldb = (uint32_t)ld * 2;
  if (PAD) zero_tiles<NT>(smem, 2 * (KT + VT), tid);
  BlockDma<BSW, DH, NT> dma;
  dma.init(wave, lane, PAD ? dh : DH);
  dma.template issue<PAD>(rk, smem, ldb, 0, seq - 1, wave);
  dma.template issue<PAD>(rv, smem + KT, ldb, 0, seq - 1, wave);
  __builtin_amdgcn_s_waitcnt(kWaitAllLoads);
  __syncthreads();
  for (int blk = 0; blk < nblk; ++blk) {
    const bf16_t* kt_ = smem + (blk & 1) * (KT + VT);
    const bf16_t* vt_ = kt_ + KT;
    if (blk + 1 < nblk) {
      bf16_t* nxt = smem + ((blk + 1) & 1) * (KT + VT);
      dma.template issue<PAD>(rk, nxt, ldb, (blk + 1) * BSW, seq - 1, wave);
      dma.template issue<PAD>(rv, nxt + KT, ldb, (blk + 1) * BSW, seq - 1, wave);
    }
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
      const int trow = WK * kg + 32 * kt;   // tile row of this 32-key tile
      const int k0 = blk * BSW + trow;      // its first key
      if (k0 >= seq || (causal && k0 > qw0 + 31)) continue;
      f32x16 s, dp;
      zero(s);
      zero(dp);
#pragma unroll
      for (int ks = 0; ks < DH / 16; ++ks) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(kt_, trow, 16 * ks, lane), qf[ks], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(vt_, trow, 16 * ks, lane), dof[ks], dp, 0, 0, 0);
      }
      if ((causal && k0 + 31 > qw0) || (k0 + 32 > seq)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 8 * (r >> 2) + 4 * hl + (r & 3);
          const bool dead = key >= seq || (causal && key > qrow);
          const float p = dead ? 0.f : __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, -lse2));
          s[r] = p * (dp[r] - dl);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, -lse2)) * (dp[r] - dl);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 dsb = acc_to_frag(s, t);
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
          acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<DH>(kt_, 32 * dt, trow + 16 * t, lane), dsb, acc[dt],
                                                            0, 0, 0);
      }
    }
    __builtin_amdgcn_s_waitcnt(kWaitAllLoads);
    __syncthreads();
  }
  if (KW > 1) {
    constexpr int SLOT = (DH / 2) * 64;  // [DH/2 registers][64 lanes] fp32
    static_assert((size_t)QW * (KW - 1) * SLOT * 4 <= (size_t)2 * (KT + VT) * 2, "merge slots must fit in the tiles");
    float* slots = reinterpret_cast<float*>(smem);
    if (kg > 0) {
      float* my = slots + ((kg - 1) * QW + qg) * SLOT;
#pragma unroll
      for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) my[(dt * 16 + r) * 64 + lane] = acc[dt][r];
    }
    __syncthreads();
    if (kg > 0) return;
#pragma unroll 1
    for (int g = 1; g < KW; ++g) {
      const float* other = slots + ((g - 1) * QW + qg) * SLOT;
#pragma unroll
      for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] += other[(dt * 16 + r) * 64 + lane];
    }
  }
  if (qrow < seq) {
    bf16_t* row = dq + ((size_t)b * seq + qrow) * h + (size_t)head * dh;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt) store_tile_t(row + 32 * dt, acc[dt], scale, lane, PAD ? dh - 32 * dt : 32);
  }
}

// Backward, dK and dV.  A workgroup owns 32 KG keys of one head and streams blocks of 32 QG queries
// (Q and dO tiles plus their log-sum-exp and delta).  Each (key group, query group) pair is served
// by TWO waves with different roles, which halves the accumulators a wave has to hold:
//   role 0 keeps K:  S = Q K^T,  P = exp2(S scale - lse),  dV^T += dO^T P;   hands P over through LDS;
//   role 1 keeps V:  dP = dO V^T,  dS = P (dP - delta),     dK^T += Q^T dS.
// Both roles run the same two matrix products per tile (one against Q, one against dO); only the
// elementwise step between them differs.  The QG partial sums of a key group are added in
// query-group order through LDS at the end and written in place over K and V (a key block is read
// only by its own workgroup).
template <int DH, int KG, int QG, bool PAD>
__global__ __launch_bounds__(KG * QG * 128, KG * QG == 2 ? 3 : 1) void attn_bwd_dkv_mfma(
    int seq, int heads, int dh, int causal, const bf16_t* qkv, const float* __restrict__ lse, const float* __restrict__ delta,
    const bf16_t* __restrict__ d_o, bf16_t* dqkv, float scale, float scale_log2) {
  constexpr int NP = KG * QG, NT = NP * 128, BK = 32 * KG, BSQ = 32 * QG;
  constexpr int QT = BSQ * DH;
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];  // [2][Q tile | dO tile], stats, P exchange
  float* stats = reinterpret_cast<float*>(smem + 4 * QT);       // [2][lse2[BSQ] | delta[BSQ]]
  float* xch = stats + 4 * BSQ;                                  // [NP][16 registers][64 lanes]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hl = lane >> 5;
  const int role = wave / NP, pair = wave % NP, kg = pair % KG, qg = pair / KG;
  // grid = (heads * batch, key blocks): early key blocks see the most queries and go first
  const int h = heads * dh, head = blockIdx.x % heads, b = blockIdx.x / heads;
  const int k0 = blockIdx.y * BK, kw0 = k0 + 32 * kg, krow = kw0 + (lane & 31);
  const size_t ld = (size_t)3 * h;
  const bf16_t* base = qkv + (size_t)b * seq * ld + (size_t)head * dh;
  const bf16_t* dob = d_o + (size_t)b * seq * h + (size_t)head * dh;
  const float* lse_b = lse + ((size_t)b * heads + head) * seq;
  const float* delta_b = delta + ((size_t)b * heads + head) * seq;

  bf16x8 kvf[DH / 16];  // role 0: K rows of this key group; role 1: V rows
  {
    const bf16_t* kp = base + (size_t)min(krow, seq - 1) * ld + (role ? 2 * h : h);
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) kvf[ks] = load_frag(kp, 16 * ks + 8 * hl, PAD ? dh : DH);
  }
  f32x16 acc[DH / 32];  // role 0: dV^T, role 1: dK^T (unscaled)
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt) zero(acc[dt]);
  const int qstart = causal ? (k0 / BSQ) * BSQ : 0;
  const int nblk = (seq - qstart + BSQ - 1) / BSQ;
  const i32x4 rq = make_rsrc(base), rdo = make_rsrc(dob);
  const uint32_t ldb = (uint32_t)ld * 2, hb = (uint32_t)h * 2;
  if (PAD) zero_tiles<NT>(smem, 4 * QT, tid);
  BlockDma<BSQ, DH, NT> dma;
  dma.init(wave, lane, PAD ? dh : DH);
  float st_reg = 0.f;  // threads 0..BSQ-1: lse2 of query tid; BSQ..2 BSQ-1: delta of query tid-BSQ
  auto load_stats = [&](int q0) {
    if (tid < 2 * BSQ) {
      const int qi = q0 + (tid % BSQ);
      st_reg = qi < seq ? (tid < BSQ ? lse_b[qi] * kLog2e : delta_b[qi]) : 0.f;
    }
  };
  dma.template issue<PAD>(rq, smem, ldb, qstart, seq - 1, wave);
  dma.template issue<PAD>(rdo, smem + QT, hb, qstart, seq - 1, wave);
  load_stats(qstart);
  if (tid < 2 * BSQ) stats[tid] = st_reg;
  __builtin_amdgcn_s_waitcnt(kWaitAllLoads);
  __syncthreads();
  float* my_xch = xch + pair * (16 * 64) + lane;
  for (int blk = 0; blk < nblk; ++blk) {
    const int q0 = qstart + blk * BSQ + 32 * qg;  // the pair's 32 queries
    const int trow = 32 * qg;
    const bf16_t* qt_ = smem + (blk & 1) * 2 * QT;
    const bf16_t* dot_ = qt_ + QT;
    const bf16_t* first = role ? dot_ : qt_;    // role 0: S = Q K^T        role 1: dP = dO V^T
    const bf16_t* second = role ? qt_ : dot_;   // role 0: dV^T += dO^T P   role 1: dK^T += Q^T dS
    const float* st_ = stats + (blk & 1) * 2 * BSQ + (role ? BSQ : 0) + trow;  // lse2 (role 0) or delta (role 1)
    if (blk + 1 < nblk) {  // the other stage: every wave left it at the last barrier
      bf16_t* nxt = smem + ((blk + 1) & 1) * 2 * QT;
      dma.template issue<PAD>(rq, nxt, ldb, qstart + (blk + 1) * BSQ, seq - 1, wave);
      dma.template issue<PAD>(rdo, nxt + QT, hb, qstart + (blk + 1) * BSQ, seq - 1, wave);
      load_stats(qstart + (blk + 1) * BSQ);
    }
    const bool active = q0 < seq && (!causal || q0 + 31 >= kw0);  // the same for both waves of a pair
    f32x16 t;
    if (active) {
      zero(t);
#pragma unroll
      for (int ks = 0; ks < DH / 16; ++ks)
        t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(first, trow, 16 * ks, lane), kvf[ks], t, 0, 0, 0);
      if (role == 0) {
        if ((causal && q0 < kw0 + 31) || (q0 + 32 > seq) || (kw0 + 32 > seq)) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qi = 8 * (r >> 2) + 4 * hl + (r & 3);
            const int query = q0 + qi;
            const bool dead = query >= seq || krow >= seq || (causal && krow > query);
            t[r] = dead ? 0.f : __builtin_amdgcn_exp2f(__builtin_fmaf(t[r], scale_log2, -st_[qi]));
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qi = 8 * (r >> 2) + 4 * hl + (r & 3);
            t[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(t[r], scale_log2, -st_[qi]));
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) my_xch[r * 64] = t[r];
      }
    }
    __syncthreads();  // P of every active pair is in LDS
    if (active) {
      if (role == 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qi = 8 * (r >> 2) + 4 * hl + (r & 3);
          t[r] = my_xch[r * 64] * (t[r] - st_[qi]);
        }
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8 fb = acc_to_frag(t, tt);
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
          acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<DH>(second, 32 * dt, trow + 16 * tt, lane), fb,
                                                            acc[dt], 0, 0, 0);
      }
    }
    if (blk + 1 < nblk && tid < 2 * BSQ) stats[((blk + 1) & 1) * 2 * BSQ + tid] = st_reg;
    __builtin_amdgcn_s_waitcnt(kWaitAllLoads);
    __syncthreads();  // next tiles staged; the exchange slots may be rewritten
  }
  // Merge the query groups, one after the other so that one set of slots is enough:
  // slot of (role, key group) = [DH/2 registers][64 lanes] fp32.
  if (QG > 1) {
    constexpr int SLOT = (DH / 2) * 64;
    float* slot = reinterpret_cast<float*>(smem) + (role * KG + kg) * SLOT + lane;
#pragma unroll 1
    for (int g = 1; g < QG; ++g) {
      if (qg == g) {
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) slot[(dt * 16 + r) * 64] = acc[dt][r];
      }
      __syncthreads();
      if (qg == 0) {
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[dt][r] += slot[(dt * 16 + r) * 64];
      }
      __syncthreads();
    }
  }
  if (qg == 0 && krow < seq) {
    bf16_t* row = dqkv + ((size_t)b * seq + krow) * ld + (size_t)head * dh + (role ? h : 2 * h);
    const float mul = role ? scale : 1.0f;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt) store_tile_t(row + 32 * dt, acc[dt], mul, lane, PAD ? dh - 32 * dt : 32);
  }
}

template <int DH, int QW, int KW, int NKT, bool PAD>
int fwd_launch(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv, void* o, float* lse) {
  constexpr size_t lds = 2 * sizeof(bf16_t) * 32 * NKT * KW * 2 * DH;
  static std::atomic<bool> done{false};
  if (int rc = reserve_lds(attn_fwd_mfma<DH, QW, KW, NKT, PAD>, lds, done, "attention_forward")) return rc;
  const float scale_log2 = kLog2e / sqrtf((float)dh);
  attn_fwd_mfma<DH, QW, KW, NKT, PAD><<<dim3(heads * batch, (seq + 32 * QW - 1) / (32 * QW)), dim3(QW * KW * 64), lds, st>>>(
      seq, heads, dh, causal, (const bf16_t*)qkv, (bf16_t*)o, lse, scale_log2);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "attention_forward launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

// Few (128-query block, head) pairs: 64-query workgroups whose 8 waves split 128-key blocks four
// ways, so that every compute unit gets work; otherwise 128-query workgroups of 4 waves, each
// taking whole 64-key blocks, two workgroups to a compute unit.
// The attn_shape tuning switch (0|1|2) forces a family of launch shapes (tests and tuning).
int shape_family(int batch, int seq, int heads) {
  if (const int f = tuning(kTuneAttnShape); f >= 0) return f;
  return (long)((seq + 127) / 128) * heads * batch < 512 ? 0 : 1;
}

template <int DH, bool PAD>
int fwd_t(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv, void* o, float* lse) {
  if (shape_family(batch, seq, heads) == 0) return fwd_launch<DH, 2, 4, 1, PAD>(st, batch, seq, heads, dh, causal, qkv, o, lse);
  return fwd_launch<DH, 4, 1, 2, PAD>(st, batch, seq, heads, dh, causal, qkv, o, lse);
}

template <int DH, int QW, int KW, int NKT, int KG, int QG, bool PAD>
int bwd_launch(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv, const void* o,
               const float* lse, const void* d_o, void* dqkv, void* dq_stage, float* delta) {
  constexpr size_t lds_dq = 2 * sizeof(bf16_t) * 32 * NKT * KW * 2 * DH;
  constexpr size_t tiles_dkv =
      4 * sizeof(bf16_t) * 32 * QG * DH + (4 * 32 * QG + (size_t)KG * QG * 16 * 64) * sizeof(float);
  constexpr size_t merge_dkv = QG > 1 ? (size_t)2 * KG * (DH / 2) * 64 * sizeof(float) : 0;
  constexpr size_t lds_dkv = tiles_dkv > merge_dkv ? tiles_dkv : merge_dkv;
  static_assert(lds_dq <= 160 * 1024 && lds_dkv <= 160 * 1024, "tiles exceed the LDS of a compute unit");
  static std::atomic<bool> done_dq{false}, done_dkv{false};
  if (int rc = reserve_lds(attn_bwd_dq_mfma<DH, QW, KW, NKT, PAD>, lds_dq, done_dq, "attention_backward")) return rc;
  if (int rc = reserve_lds(attn_bwd_dkv_mfma<DH, KG, QG, PAD>, lds_dkv, done_dkv, "attention_backward")) return rc;
  const float scale = 1.0f / sqrtf((float)dh), scale_log2 = kLog2e * scale;
  attn_bwd_dq_mfma<DH, QW, KW, NKT, PAD><<<dim3(heads * batch, (seq + 32 * QW - 1) / (32 * QW)), dim3(QW * KW * 64), lds_dq, st>>>(
      seq, heads, dh, causal, (const bf16_t*)qkv, (const bf16_t*)o, lse, (const bf16_t*)d_o, (bf16_t*)dq_stage, delta, scale,
      scale_log2);
  attn_bwd_dkv_mfma<DH, KG, QG, PAD><<<dim3(heads * batch, (seq + 32 * KG - 1) / (32 * KG)), dim3(KG * QG * 128), lds_dkv, st>>>(
      seq, heads, dh, causal, (const bf16_t*)qkv, lse, delta, (const bf16_t*)d_o, (bf16_t*)dqkv, scale, scale_log2);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMC_ERR_HIP, "attention_backward launch failed: %s", hipGetErrorString(e));
  return PMC_OK;
}

template <int DH, bool PAD>
int bwd_t(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv, const void* o, const float* lse,
          const void* d_o, void* dqkv, void* dq_stage, float* delta) {
  const int fam = shape_family(batch, seq, heads);
  if (fam == 0)
    return bwd_launch<DH, 2, 4, 1, 2, 2, PAD>(st, batch, seq, heads, dh, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta);
  if (fam == 2)
    return bwd_launch<DH, 4, 1, 2, 4, 1, PAD>(st, batch, seq, heads, dh, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta);
  return bwd_launch<DH, 4, 1, 2, 2, 1, PAD>(st, batch, seq, heads, dh, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta);
}

int check(const char* what, int batch, int seq, int heads, int dh, const void* qkv) {
  if (batch <= 0 || seq <= 0 || heads <= 0) return fail(PMC_ERR_INVALID, "%s: batch=%d seq=%d heads=%d", what, batch, seq, heads);
  if (dh < 8 || dh > 128 || dh % 8)
    return fail(PMC_ERR_INVALID, "%s: matrix-core path needs a head size that is a multiple of 8 up to 128, got %d", what, dh);
  if (seq > 65535 * 32 || (long)heads * batch > 0x7fffffffL) return fail(PMC_ERR_INVALID, "%s: seq or heads*batch exceed the grid limit", what);
  if (reinterpret_cast<uintptr_t>(qkv) & 15) return fail(PMC_ERR_INVALID, "%s: qkv must be 16-byte aligned", what);
  // the tile loads address one sequence's rows with 32-bit byte offsets inside a 2 GB window
  if ((size_t)seq * 3 * heads * dh * 2 > 0x7fffffffull)
    return fail(PMC_ERR_INVALID, "%s: one sequence's q|k|v rows (%d x %d) exceed 2 GB", what, seq, 3 * heads * dh);
  return PMC_OK;
}

}  // namespace

// Head sizes 64 and 128 fill the kernels' tiles; the other multiples of 8 run in the next larger
// tile with its remaining columns held at zero.
int attention_forward_mfma(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv, void* o,
                           float* lse) {
  if (int rc = check("attention_forward", batch, seq, heads, dh, qkv)) return rc;
  if (reinterpret_cast<uintptr_t>(o) & 15) return fail(PMC_ERR_INVALID, "attention_forward: o must be 16-byte aligned");
  if (dh == 64) return fwd_t<64, false>(st, batch, seq, heads, dh, causal, qkv, o, lse);
  if (dh == 128) return fwd_t<128, false>(st, batch, seq, heads, dh, causal, qkv, o, lse);
  if (dh < 64) return fwd_t<64, true>(st, batch, seq, heads, dh, causal, qkv, o, lse);
  return fwd_t<128, true>(st, batch, seq, heads, dh, causal, qkv, o, lse);
}

int attention_backward_mfma(hipStream_t st, int batch, int seq, int heads, int dh, int causal, const void* qkv,
                            const void* o, const float* lse, const void* d_o, void* dqkv, void* dq_stage, float* delta) {
  if (int rc = check("attention_backward", batch, seq, heads, dh, qkv)) return rc;
  if ((reinterpret_cast<uintptr_t>(o) | reinterpret_cast<uintptr_t>(d_o) | reinterpret_cast<uintptr_t>(dqkv) |
       reinterpret_cast<uintptr_t>(dq_stage)) & 15)
    return fail(PMC_ERR_INVALID, "attention_backward: tensors must be 16-byte aligned");
  if (dh == 64) return bwd_t<64, false>(st, batch, seq, heads, dh, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta);
  if (dh == 128) return bwd_t<128, false>(st, batch, seq, heads, dh, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta);
  if (dh < 64) return bwd_t<64, true>(st, batch, seq, heads, dh, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta);
  return bwd_t<128, true>(st, batch, seq, heads, dh, causal, qkv, o, lse, d_o, dqkv, dq_stage, delta);
}

}  // namespace k
}  // namespace pmc
