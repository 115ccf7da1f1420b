// Expert FFN of Eq. 1 as two grouped GEMMs over the send buffer's expert segments:
//   H = GeLU(S_e . W_in[e]^T)   (rows x h, rounded once to bf16)
//   O = H . W_out[e]^T          (rows x d, rounded once to the storage type)
// Both weights are stored row-major in Eq. 1's orientation ([h,d] and [d,h]), so both GEMMs
// contract over the contiguous axis of both operands ("NT" form): every MFMA fragment is one
// 16-byte LDS read.  bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// Kernels that share the operand orientation and the epilogue:
//   ffn_gemm_generic         any shape the descriptor allows, fp32 or bf16 activations (fallback)
//   ffn_gemm_256             256x256x64 tiles, register-staged double buffer, row-major weights
//   ffn_gemm_dma_persistent  256x256x32 tiles, LDS rings filled by direct-to-LDS loads, weights pre-packed
//                            by locmoe_pack_weights into the LDS image of each k-step; four waves with the
//                            accumulators in the accumulation registers; one work-group per compute unit
//                            works through a queue of tiles (expert counts that are multiples of 8, up to 512)
//   ffn_gemm_dma             the same pipeline with one tile per work-group (other expert counts)
//
// The weight rows feed the MFMA's A operand and the activation rows its B operand, i.e. the
// tile is computed transposed (D[n][m]); a lane then owns 4 consecutive output columns n of one
// row m per accumulator quad and stores them as one 8-byte (bf16) or 16-byte (fp32) vector.
#include <math.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

#include "common.h"
#include "gelu_coef.h"

namespace locmoe {
namespace {

// GeLU for outputs that are rounded to bf16: GeLU(v) = max(v,0) - |v| Phi(-|v|), with
// 2 Phi(-x) = exp2(q(x)), q the degree-6 polynomial of gelu_coef.h on [0, 6] (argument clamped: the
// tail beyond is below 6e-9).  Relative error below 5e-5, absolute below 7e-6: forty times finer than
// the bf16 rounding that follows, at 10 vector ops and one transcendental per value (a rational erfc
// form with the same tail behaviour costs 15 and two; the epilogue's vector work was a tenth of the
// first GEMM's time with it).
// max(v,0) is formed as (v + |v|)/2 so that a NaN input stays a NaN.
__device__ __forceinline__ float gelu_bf16(float v) {
  const float x = fminf(fabsf(v), kGeluXMax);
  float q = kGeluCoef[kGeluDegree];
#pragma unroll
  for (int k = kGeluDegree - 1; k >= 0; --k) q = fmaf(q, x, kGeluCoef[k]);
  return 0.5f * fmaf(-x, __builtin_amdgcn_exp2f(q), v + fabsf(v));
}

__device__ __forceinline__ f32x16 mfma_bf16(const bf16x8& a, const bf16x8& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// GeLU'(v) = Phi(v) + v phi(v) for factors of outputs that are rounded to bf16, from the same polynomial:
// Phi(-|v|) = exp2(q(|v|)) / 2 (absolute error below 2.3e-5), phi(v) = exp2(-v^2 log2(e)/2) / sqrt(2 pi).
__device__ __forceinline__ float gelu_grad_bf16(float v) {
  const float x = fminf(fabsf(v), kGeluXMax);
  float q = kGeluCoef[kGeluDegree];
#pragma unroll
  for (int k = kGeluDegree - 1; k >= 0; --k) q = fmaf(q, x, kGeluCoef[k]);
  const float tail = 0.5f * __builtin_amdgcn_exp2f(q);  // Phi(-|v|)
  const float Phi = v >= 0.f ? 1.0f - tail : tail;
  const float phi = 0.3989422804f * __builtin_amdgcn_exp2f(-0.7213475204f * v * v);
  return fmaf(v, phi, Phi);
}

// What happens to an accumulator on its way to memory
constexpr int kEpiNone = 0;      // rounded and stored
constexpr int kEpiGelu = 1;      // GeLU, then rounded and stored (H of Eq. 1)
constexpr int kEpiGeluSave = 2;  // the same, and the pre-activation Z is stored (bf16) to `aux` for the backward
constexpr int kEpiGeluGrad = 3;  // multiplied by GeLU'(Z), Z read from `aux` (bf16): dZ = dH * GeLU'(Z)

// One accumulator quad -> memory.  q holds D[n0..n0+3][m] for one row m.
template <int EPI, bool OUT_F32>
__device__ __forceinline__ void store_quad(void* C, uint16_t* aux, size_t row, int ldc, int n0, float q0, float q1,
                                           float q2, float q3) {
  static_assert(!(EPI != kEpiNone && OUT_F32), "the hidden activations and their gradients are stored as bf16");
  if (EPI == kEpiGeluSave) *(uint2*)(aux + row * ldc + n0) = make_uint2(pack_bf16x2(q0, q1), pack_bf16x2(q2, q3));
  if (EPI == kEpiGelu || EPI == kEpiGeluSave) {
    q0 = gelu_bf16(q0); q1 = gelu_bf16(q1); q2 = gelu_bf16(q2); q3 = gelu_bf16(q3);
  }
  if (EPI == kEpiGeluGrad) {
    const uint2 z = *(const uint2*)(aux + row * ldc + n0);
    q0 *= gelu_grad_bf16(bf16_bits_to_f32(z.x & 0xFFFFu));
    q1 *= gelu_grad_bf16(__uint_as_float(z.x & 0xFFFF0000u));
    q2 *= gelu_grad_bf16(bf16_bits_to_f32(z.y & 0xFFFFu));
    q3 *= gelu_grad_bf16(__uint_as_float(z.y & 0xFFFF0000u));
  }
  if (OUT_F32) {
    *(float4*)((float*)C + row * ldc + n0) = make_float4(q0, q1, q2, q3);
  } else {
    *(uint2*)((uint16_t*)C + row * ldc + n0) = make_uint2(pack_bf16x2(q0, q1), pack_bf16x2(q2, q3));
  }
}

// ---------------------------------------------------------------------------------------------
// Generic kernel: 64x64x32 tile, 4 waves, any K and N that are multiples of 8, fp32 or bf16
// activations.  Correct for every shape the descriptor allows; not tuned.
// ---------------------------------------------------------------------------------------------
constexpr int kGenThreads = 256;
constexpr int kGenLd = 40;  // LDS row stride in bf16 elements (32 + 8 pad), 80 bytes

template <bool A_F32, int EPI, bool OUT_F32>
__global__ __launch_bounds__(kGenThreads) void ffn_gemm_generic(const void* __restrict__ A,
                                                                const uint16_t* __restrict__ W,
                                                                void* __restrict__ Cout, uint16_t* aux,
                                                                const int32_t* __restrict__ seg_off,
                                                                const int32_t* __restrict__ buf_expert, int Kdim,
                                                                int Ndim, int MT) {
  __shared__ __attribute__((aligned(16))) uint16_t As[64 * kGenLd];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[64 * kGenLd];
  const int r = blockIdx.y / MT, mt = blockIdx.y % MT;
  const int seg0 = seg_off[r], rows = seg_off[r + 1] - seg0;
  const int m0 = mt * 64;
  if (m0 >= rows) return;
  const int e = buf_expert[r];
  const int n0 = blockIdx.x * 64;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int lrow = tid >> 2, lch = tid & 3;
  const size_t arow = (size_t)seg0 + min(m0 + lrow, rows - 1);       // clamped: tail rows re-read the last row
  const size_t wrow = (size_t)e * Ndim + min(n0 + lrow, Ndim - 1);
  const int wm = wave >> 1, wn = wave & 1;
  f32x16 acc = {0};
  for (int k0 = 0; k0 < Kdim; k0 += 32) {
    const int kk = k0 + lch * 8;
    uint4 av = make_uint4(0, 0, 0, 0), bv = make_uint4(0, 0, 0, 0);
    if (kk < Kdim) {
      if (A_F32) {
        const float4* p = (const float4*)((const float*)A + arow * Kdim + kk);
        const float4 f0 = p[0], f1 = p[1];
        av = make_uint4(pack_bf16x2(f0.x, f0.y), pack_bf16x2(f0.z, f0.w), pack_bf16x2(f1.x, f1.y),
                        pack_bf16x2(f1.z, f1.w));
      } else {
        av = *(const uint4*)((const uint16_t*)A + arow * Kdim + kk);
      }
      bv = *(const uint4*)(W + wrow * Kdim + kk);
    }
    __syncthreads();
    *(uint4*)(As + lrow * kGenLd + lch * 8) = av;
    *(uint4*)(Bs + lrow * kGenLd + lch * 8) = bv;
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int ko = ks * 16 + (lane >> 5) * 8;
      const bf16x8 xa = *(const bf16x8*)(As + (wm * 32 + (lane & 31)) * kGenLd + ko);
      const bf16x8 wb = *(const bf16x8*)(Bs + (wn * 32 + (lane & 31)) * kGenLd + ko);
      acc = mfma_bf16(wb, xa, acc);  // D[n][m]
    }
  }
  const int m = m0 + wm * 32 + (lane & 31);
  if (m < rows) {
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int n = n0 + wn * 32 + vq * 8 + (lane >> 5) * 4;
      if (n < Ndim)  // Ndim % 8 == 0 and n % 4 == 0: the quad is entirely inside or outside
        store_quad<EPI, OUT_F32>(Cout, aux, (size_t)seg0 + m, Ndim, n, acc[vq * 4 + 0], acc[vq * 4 + 1],
                                  acc[vq * 4 + 2], acc[vq * 4 + 3]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Tuned kernel: 256x256x64 tile, 8 waves (2 along m x 4 along n, 128x64 per wave), double
// buffered LDS (2 x 64 KiB), XOR-swizzled 16-byte slots (slot = chunk ^ (row/2 mod 8): 16 lanes
// reading 16 consecutive rows touch all 64 banks once), bf16 activations, K % 64 == 0, N % 256 == 0.  Work-group ids are remapped so that each XCD (ids congruent mod 8 land on one
// XCD and share its L2) walks a contiguous range of experts, with the m-tiles that share a
// weight tile adjacent in time.
// ---------------------------------------------------------------------------------------------
constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kFastThreads = 512;
constexpr int kStageBytes = (kBM + kBN) * kBK * 2;  // 64 KiB
constexpr int kFastSmem = 2 * kStageBytes;

template <int SH>
__device__ __forceinline__ int swz(int row, int chunk) { return (chunk ^ ((row >> SH) & 7)) << 4; }

template <int EPI, bool OUT_F32, int SH>
__global__ __launch_bounds__(kFastThreads) void ffn_gemm_256(const uint16_t* __restrict__ A,
                                                             const uint16_t* __restrict__ W,
                                                             void* __restrict__ Cout, uint16_t* aux,
                                                             const int32_t* __restrict__ seg_off,
                                                             const int32_t* __restrict__ buf_expert, int Kdim,
                                                             int Ndim, int MT, int NT, int total) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int id = blockIdx.x;
  const int lin = (total % 8 == 0) ? (id % 8) * (total / 8) + id / 8 : id;
  const int mt = lin % MT, nt = (lin / MT) % NT, r = lin / (MT * NT);
  const int seg0 = seg_off[r], rows = seg_off[r + 1] - seg0;
  const int m0 = mt * kBM;
  if (m0 >= rows) return;
  const int e = buf_expert[r];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave >> 2, wn = wave & 3;

  // global -> LDS assignment: 4 A chunks and 4 B chunks of 16 bytes per thread and stage
  const uint16_t* ga[4];
  const uint16_t* gb[4];
  int lds_w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + i * kFastThreads;
    const int row = c >> 3, kc = c & 7;
    ga[i] = A + ((size_t)seg0 + min(m0 + row, rows - 1)) * Kdim + kc * 8;
    gb[i] = W + ((size_t)e * Ndim + (size_t)nt * kBN + row) * Kdim + kc * 8;
    lds_w[i] = row * (kBK * 2) + swz<SH>(row, kc);
  }
  // LDS -> fragment addresses (byte offsets inside a stage, without the k-chunk part)
  const int khalf = lane >> 5;
  int a_row[4], b_row[2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) a_row[mi] = wm * 128 + mi * 32 + (lane & 31);
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) b_row[ni] = wn * 64 + ni * 32 + (lane & 31);

  f32x16 acc[2][4];
#pragma unroll
  for (int ni = 0; ni < 2; ++ni)
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) acc[ni][mi] = (f32x16){0};

  // The staging registers are native vectors and the loop body has no conditionals: the prefetch
  // of the tile after the last one is clamped to the last tile (redundant, never consumed).  With
  // branches around the prefetch the compiler demotes these arrays to scratch memory and
  // serialises every load.
  u32x4 ra[4], rb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { ra[i] = *(const u32x4*)(ga[i]); rb[i] = *(const u32x4*)(gb[i]); }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    *(u32x4*)(smem + lds_w[i]) = ra[i];
    *(u32x4*)(smem + kBM * kBK * 2 + lds_w[i]) = rb[i];
  }
  __syncthreads();

  const int KT = Kdim / kBK;
  for (int kt = 0; kt < KT; ++kt) {
    {
      const int ko = min(kt + 1, KT - 1) * kBK;
#pragma unroll
      for (int i = 0; i < 4; ++i) { ra[i] = *(const u32x4*)(ga[i] + ko); rb[i] = *(const u32x4*)(gb[i] + ko); }
    }
    const char* sa = smem + (kt & 1) * kStageBytes;
    const char* sb = sa + kBM * kBK * 2;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int kc = ks * 2 + khalf;
      bf16x8 fa[4], fb[2];
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) fb[ni] = *(const bf16x8*)(sb + b_row[ni] * (kBK * 2) + swz<SH>(b_row[ni], kc));
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) fa[mi] = *(const bf16x8*)(sa + a_row[mi] * (kBK * 2) + swz<SH>(a_row[mi], kc));
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) acc[ni][mi] = mfma_bf16(fb[ni], fa[mi], acc[ni][mi]);
    }
    {
      char* da = smem + ((kt + 1) & 1) * kStageBytes;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *(u32x4*)(da + lds_w[i]) = ra[i];
        *(u32x4*)(da + kBM * kBK * 2 + lds_w[i]) = rb[i];
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int m = m0 + wm * 128 + mi * 32 + (lane & 31);
    if (m < rows) {
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int n = nt * kBN + wn * 64 + ni * 32 + vq * 8 + khalf * 4;
          store_quad<EPI, OUT_F32>(Cout, aux, (size_t)seg0 + m, Ndim, n, acc[ni][mi][vq * 4 + 0],
                                    acc[ni][mi][vq * 4 + 1], acc[ni][mi][vq * 4 + 2], acc[ni][mi][vq * 4 + 3]);
        }
    }
  }
}


// ---------------------------------------------------------------------------------------------
// DMA kernels: 256x256 tile, k-steps of 32 taken two at a time ("double steps"), four waves, one per
// SIMD (2 along m x 2 along n, 128x128 per wave, the 256 accumulators in the accumulation registers).
// Both operands reach LDS by direct-to-LDS loads (global_load_lds_dwordx4: no staging registers, no
// ds_write), in two rings that fill all 160 KiB of a CU:
//   weights      3 slots x 32 KiB, one double step each: two consecutive 16 KiB blocks of the packed
//                layout (256 rows x 64 B each), so a work-group's weight stream is one contiguous run;
//   activations  2 slots x 32 KiB, one double step each (256 rows x 128 B): rows are fetched as whole
//                128-byte lines (with 64-byte row segments every line was requested in two consecutive
//                k-steps: +5 % from whole lines alone).
// Weights come from HBM and are issued two double steps ahead, activations mostly from L2 and one ahead.
//
// A direct-to-LDS load writes lane l's 16 bytes at base + 16 l, so the LDS image is produced by
// choosing which global chunk each lane fetches.  Slot functions (measured conflict-free for the
// 16x16x32 fragment read, lane l: row l%16, chunk l/16): 64-byte weight rows: chunk ^ (row/2 mod 4);
// 128-byte activation rows: chunk ^ (row/2 mod 8).
//
// One barrier per double step D, between the two MFMA groups of its second k-step.  By then every wave
// has issued all its fragment reads of double step D, so behind the barrier the slots of W(D) and A(D)
// are refilled: A(D+2) at once, W(D+3) during the next k-step (a slot ahead of need either way).  The
// barrier also publishes W(D+1) and A(D+1), whose first fragments are read right behind it.
// The compiler does not know about these loads (inline asm), so the vmcnt accounting is explicit:
// direct-to-LDS loads complete in order and nothing else in the K loop uses vmcnt.  Per wave a double
// step issues 8 weight and 8 activation copies; at the barrier of D everything issued after A(D+1) is
// the 8 copies of W(D+2), hence vmcnt(8).
//
// Rows of the tile are owned in interleaved 16-row subtiles (wave row wm owns subtiles wm, wm+2,
// ...), so a ragged tile skips MFMAs evenly across waves, at 32-row granularity overall.
// ---------------------------------------------------------------------------------------------
constexpr int kDmaBK = 32;
constexpr int kDmaWaves = 4;               // one wave per SIMD
constexpr int kDmaThreads = kDmaWaves * 64;
constexpr int kPackBlock = kBN * kDmaBK * 2;                    // 16 KiB: one packed weight block (one k-step)
constexpr int kWSlots = 3, kWSlotBytes = 2 * kPackBlock;        // 3 x 32 KiB
constexpr int kASlots = 2, kASlotBytes = kBM * kDmaBK * 2 * 2;  // 2 x 32 KiB
constexpr int kWRing = kASlots * kASlotBytes;                   // weights ring starts after the activations ring
constexpr int kDmaSmem = kWRing + kWSlots * kWSlotBytes;        // 160 KiB: the whole LDS of a CU

// v_mfma_f32_16x16x32_bf16 with the accumulator pinned to accumulation registers and updated in place.  With all 256
// of them holding accumulators the compiler's own register assignment routes most MFMAs through a spare
// tuple (four copies per MFMA); written this way there are none.  The compiler does not see an MFMA here,
// so it inserts none of the wait states an MFMA needs around other instructions; the places that need
// them are handled by hand: the results are read only after explicit wait states behind the K loop; the
// accumulators are never zeroed by register writes (an MFMA that follows such a write too closely reads
// the old value: seen as wrong last components of some accumulators) but by MFMAs of a zero operand, and
// that operand is pinned behind wait states of its own (without them: NaNs).
template <bool FROM_ZERO>
__device__ __forceinline__ void mfma16_acc(f32x4& c, const bf16x8& a, const bf16x8& b) {
  if (FROM_ZERO)  // c = a.b + 0
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=a"(c) : "v"(a), "v"(b));
  else            // c += a.b
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// What the pipeline needs to know about one 256x256 output tile (all wave-uniform).
struct DmaTile {
  const char* Abase;   // first activation row of the tile
  const char* Wbase;   // first packed block of the tile's 256 weight rows (output columns)
  int rows_left;       // live rows from the tile's first row to the segment's end (>= 1)
  size_t crow0;        // first output row
  int n_base;          // first output column
};
// Ring positions, carried from tile to tile: the slots of the current double step's weights and activations.
struct DmaRing { int wcur, acur; };
// What a lane contributes to the activation copies.  Lane l of the copy of row block b (8 rows x 128 B)
// fetches row 8 b + l/8; LDS chunk l%8 receives source chunk (l%8) ^ (row/2 mod 8), which is the same for
// all of a wave's blocks (they are 32 rows apart).  Rows past the segment's end re-read its last row
// (results masked at the store).
struct DmaLane {
  uint32_t row0;       // row of this lane in the wave's first block
  uint32_t chunk16;    // byte offset of its source chunk inside a 128-byte row segment
  uint32_t row_bytes;  // bytes per activation row
  uint32_t row0q;      // the K loop's assignment of blocks to waves: row of this lane in block 4 wave
  uint32_t chunk16q;   // ... and its source chunk there (blocks 4 wave + odd: chunk16q ^ 64)
};
__device__ __forceinline__ DmaLane make_lane(int Kdim, int wave, int lane) {
  const uint32_t row0 = 8 * wave + (lane >> 3);
  const uint32_t row0q = 32 * wave + (lane >> 3);
  return DmaLane{row0, (uint32_t)(((lane & 7) ^ ((row0 >> 1) & 7)) * 16), (uint32_t)Kdim * 2u, row0q,
                 (uint32_t)(((lane & 7) ^ ((row0q >> 1) & 7)) * 16)};
}

// `span` = rows per m-tile of this segment (at most 256; the segment's last tile may hold fewer)
__device__ __forceinline__ DmaTile make_tile(const uint16_t* A, const uint16_t* Wp, int seg0, int rows, int span,
                                             int mt, int nt, int e, int Kdim, int Ndim) {
  DmaTile t;
  const int m0 = mt * span;
  t.rows_left = min(rows - m0, span);
  t.Abase = (const char*)(A + ((size_t)seg0 + m0) * Kdim);
  t.Wbase = (const char*)(Wp + ((size_t)e * Ndim + (size_t)nt * kBN) * (size_t)Kdim);
  t.crow0 = (size_t)seg0 + m0;
  t.n_base = nt * kBN;
  return t;
}
// Stand-in for "the tile after the last": prefetches past the end of `t` re-read its own last two double
// steps, which nobody consumes.
__device__ __forceinline__ DmaTile tail_alias(const DmaTile& t, int KD) {
  DmaTile a = t;
  a.Wbase = t.Wbase + (size_t)(KD - 2) * kWSlotBytes;
  a.Abase = t.Abase + (size_t)(KD - 2) * (kDmaBK * 4);
  return a;
}

// copy i (of this wave's eight) of the weights of double step D into ring slot `slot`: 1 KiB block wave + 4 i of 32
__device__ __forceinline__ void issue_w1(const char* wbase, int D, int slot, int i, uint32_t lds0, int wave,
                                         int lane) {
  const char* wb = wbase + (size_t)D * kWSlotBytes;
  const uint32_t blk = (uint32_t)(wave + kDmaWaves * i) * 1024;
  dma_1k(wb, blk + lane * 16, lds0 + kWRing + (uint32_t)slot * kWSlotBytes + blk);
}
// copy j (of this wave's eight) of the activations of double step D into ring slot `slot`: block wave + 4 j of
// 32, a block being 8 rows x 128 B
__device__ __forceinline__ void issue_a1(const DmaTile& t, const DmaLane& ln, int D, int slot, int j, uint32_t lds0,
                                         int wave) {
  const uint32_t row = min(ln.row0 + 32u * j, (uint32_t)t.rows_left - 1u);
  dma_1k(t.Abase + (size_t)D * (kDmaBK * 4), row * ln.row_bytes + ln.chunk16,
         lds0 + (uint32_t)slot * kASlotBytes + (wave + kDmaWaves * j) * 1024);
}

// The K loop's copies.  There a wave owns blocks 16 g + 4 wave + sub (g = 0, 1; sub = 0..3) of a slot instead of
// blocks wave + 4 i: the four blocks of a group are consecutive KiB of LDS, so one M0 write serves four copies
// (the loop has one wave per SIMD and issues in order: every instruction between two MFMAs costs MFMA time).
// c = 4 g + sub.  For the weights source and destination advance together; for the activations the immediate is
// taken off the lane's offset again (from a base 4 KiB below the rows, so that the offset stays non-negative).
__device__ __forceinline__ void issue_w1q(const char* wbase, int D, int slot, int c, uint32_t lds0, int wave, int lane) {
  const uint32_t grp = (uint32_t)(c >> 2) * 16384u + (uint32_t)wave * 4096u;
  if ((c & 3) == 0) dma_base(lds0 + kWRing + (uint32_t)slot * kWSlotBytes + grp);
  dma_1k_sub(wbase + (size_t)D * kWSlotBytes, grp + lane * 16, c & 3);
}
__device__ __forceinline__ void issue_a1q(const DmaTile& t, const DmaLane& ln, int D, int slot, int c, uint32_t lds0,
                                          int wave) {
  const uint32_t sub = (uint32_t)(c & 3);
  if (sub == 0) dma_base(lds0 + (uint32_t)slot * kASlotBytes + (uint32_t)(c >> 2) * 16384u + (uint32_t)wave * 4096u);
  const uint32_t row = min(ln.row0q + 128u * (uint32_t)(c >> 2) + 8u * sub, (uint32_t)t.rows_left - 1u);
  dma_1k_sub(t.Abase + (size_t)D * (kDmaBK * 4) - 4096, row * ln.row_bytes + (ln.chunk16q ^ ((sub & 1u) << 6)) + 4096u - sub * 1024u,
             (int)sub);
}

// Fills the pipeline for the first tile of a work-group: A(0) W(0) W(1) A(1), all landed and visible to
// every wave on return.  Later tiles find the same state because the tile before them prefetched it.
__device__ __forceinline__ void dma_prefill(const DmaTile& t, const DmaLane& ln, DmaRing& ring, uint32_t lds0, int wave,
                                            int lane) {
  ring = DmaRing{0, 0};
#pragma unroll
  for (int D = 0; D < 2; ++D) {
#pragma unroll
    for (int j = 0; j < 8; ++j) issue_a1(t, ln, D, D, j, lds0, wave);
#pragma unroll
    for (int i = 0; i < 8; ++i) issue_w1(t.Wbase, D, D, i, lds0, wave, lane);
  }
  wait_vmcnt<0>();
  __syncthreads();
}

// One output tile.  16 fragment reads feed 64 MFMAs per k-step.  (An eight-wave form, 128x64 per wave and
// two waves per SIMD, reads 12 fragments per 32 MFMAs: half as much again in LDS traffic, and measured
// 3-4 % slower on both GEMMs.)  The K loop uses v_mfma_f32_16x16x32_bf16: one MFMA consumes a whole 32-wide
// k-step of a 16x16 output tile, and lane l always reads LDS chunk l/16 of its rows.  In pure MFMA loops on
// random bf16 operands this shape sustains 1.73 PFLOP/s with one wave per SIMD (1.86 with two) against 1.64
// for the 32x32x16 shape (clock management).  With a single wave per SIMD nothing else hides the issue
// slots of the fragment reads and direct-to-LDS copies, so they are interleaved one by one between the MFMAs.
//
// On entry W(0), W(1), A(0) of `cur` have landed and are published and A(1) is in flight or landed; the
// loop's prefetches run on into `nxt`, so on exit the same holds for `nxt`, and this tile's stores may
// still be in flight: the caller drains everything with vmcnt(0) before the next tile (stores and
// direct-to-LDS loads do not retire in order relative to each other, so no smaller count is safe there).
template <int NJ, int EPI, class F>
__device__ __forceinline__ void dma_tile(const DmaTile& cur, const DmaTile& nxt, const DmaLane& ln, DmaRing& ring,
                                         uint16_t* __restrict__ Cout, uint16_t* aux, uint32_t lds0, int KD, int wm, int wn,
                                         int lane, int wave, int ldc, F&& before_epilogue) {
  // NJ = live 16-row activation subtiles of this wave
  constexpr int NLO = NJ < 4 ? NJ : 4;        // first group of subtiles
  constexpr int NHI = NJ - NLO;               // second group (0 for short tiles)
  const int kq = lane >> 4, l16 = lane & 15;
  lds_cptr lds = (lds_cptr)(uintptr_t)lds0;
  // subtile j of this wave: rows (2 j + wm)*16 .. +16; weight subtile ni: rows wn*128 + ni*16 .. +16.  The
  // swizzle terms do not depend on j or ni, so the per-subtile addresses are constant offsets from these.
  const int ra = wm * 16 + l16, rb = wn * 128 + l16;
  const int a_base0 = ra * 128 + ((kq ^ ((ra >> 1) & 7)) << 4);        // first k-step of a double step
  const int a_base1 = ra * 128 + (((4 + kq) ^ ((ra >> 1) & 7)) << 4);  // second
  const int b_base = kWRing + rb * 64 + ((kq ^ ((rb >> 1) & 3)) << 4);
  // The accumulators are zeroed by MFMAs (0 x 0 + 0): the hardware orders an MFMA's result against the
  // next MFMA that accumulates into it, which it does not do for a plain register write.
  f32x4 acc[8][8];
  {
    bf16x8 zero = {};
    asm volatile("s_nop 7" : "+v"(zero));  // (the zero operand is in its registers well before an MFMA reads it)
#pragma unroll
    for (int ni = 0; ni < 8; ++ni)
#pragma unroll
      for (int j = 0; j < NJ; ++j) mfma16_acc<true>(acc[ni][j], zero, zero);
  }

  bf16x8 fw[2][8], fa_lo[4], fa_hi[4];
  auto read_w = [&](int half, int ni, int wslot) {
    return *(const bf16x8 __attribute__((address_space(3)))*)(lds + (uint32_t)wslot * kWSlotBytes + half * kPackBlock +
                                                                b_base + ni * 1024);
  };
  auto read_a = [&](int half, int j, int aslot) {
    return *(const bf16x8 __attribute__((address_space(3)))*)(lds + (uint32_t)aslot * kASlotBytes +
                                                                (half ? a_base1 : a_base0) + j * 4096);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  // (wave-uniform by construction; said explicitly so that the ring arithmetic stays on the scalar unit)
  int wcur = __builtin_amdgcn_readfirstlane(ring.wcur), acur = __builtin_amdgcn_readfirstlane(ring.acur);

  // One k-step of double step D; PAR = which of its two.  On entry fw[PAR] and fa_lo hold the fragments of
  // this k-step; on exit fw[1-PAR] and fa_lo hold those of the next.
  auto step = [&](auto par_, auto tail_, int D) {
    constexpr int PAR = decltype(par_)::value;
    constexpr int NPAR = 1 - PAR;
    constexpr bool TAIL = decltype(tail_)::value;  // one of the tile's last two double steps
    // (register copies that the compiler may place at a loop boundary are vector writes too: keep them a few
    // wait states away from the MFMAs that read the fragments)
    asm volatile("s_nop 3" ::: "memory");
    // first group of subtiles; the second group's activation fragments are read in between
#pragma unroll
    for (int j = 0; j < NLO; ++j) {
      if (j < NHI) fa_hi[j] = read_a(PAR, 4 + j, acur);
#pragma unroll
      for (int ni = 0; ni < 8; ++ni) mfma16_acc<false>(acc[ni][j], fw[PAR][ni], fa_lo[j]);
      __builtin_amdgcn_sched_barrier(0);
    }
    const int wnext = wcur + 1 == kWSlots ? 0 : wcur + 1;
    if (PAR == 1) {
      wait_vmcnt<8>();   // W(D+1) and A(D+1) have landed (this wave's share)
      __syncthreads();   // ... and everybody's; nobody reads the slots of W(D) and A(D) any more
    }
    // second group of subtiles, with the other work spread between its MFMAs: the next k-step's fragment
    // reads first (needed soonest), then eight copies: W(D+2) in the first k-step (into the slot that the
    // previous barrier freed), A(D+2) in the second (into the slot that this barrier freed).
    // In the last two double steps the copies run on into the next tile; those steps share one pair of
    // bodies with run-time selects (a separate body per step pushed the eight loop variants out of the
    // instruction cache: -3 % on the first GEMM, whose tiles are short), the steady state has none.
    constexpr int NREAD = 8 + NLO, NITEM = NREAD + 8, NM = NHI * 8;
    const bool over = TAIL && D + 2 >= KD;
    const int Dsrc = over ? D + 2 - KD : D + 2;
    const char* wsrc = over ? nxt.Wbase : cur.Wbase;
    const int wslot2 = wnext + 1 == kWSlots ? 0 : wnext + 1;  // slot of W(D+2) = slot of W(D-1)
    const int rslot_w = PAR == 0 ? wcur : wnext;              // where the next k-step's fragments are
    const int rslot_a = PAR == 0 ? acur : acur ^ 1;
#pragma unroll
    for (int i = 0; i < NITEM; ++i) {
      if (i < 8) fw[NPAR][i] = read_w(NPAR, i, rslot_w);
      else if (i < NREAD) fa_lo[i - 8] = read_a(NPAR, i - 8, rslot_a);
      else if (PAR == 0) issue_w1q(wsrc, Dsrc, wslot2, i - NREAD, lds0, wave, lane);
      else issue_a1q(over ? nxt : cur, ln, Dsrc, acur, i - NREAD, lds0, wave);
#pragma unroll
      for (int q = i * NM / NITEM; q < (i + 1) * NM / NITEM; ++q)
        mfma16_acc<false>(acc[q & 7][4 + (q >> 3)], fw[PAR][q & 7], fa_hi[q >> 3]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (PAR == 1) {
      wcur = wnext;
      acur ^= 1;
    }
  };

#pragma unroll
  for (int ni = 0; ni < 8; ++ni) fw[0][ni] = read_w(0, ni, wcur);
#pragma unroll
  for (int j = 0; j < NLO; ++j) fa_lo[j] = read_a(0, j, acur);
  for (int D = 0; D < KD - 2; ++D) {
    step(I0{}, std::false_type{}, D);
    step(I1{}, std::false_type{}, D);
  }
#pragma nounroll
  for (int D = KD - 2; D < KD; ++D) {
    step(I0{}, std::true_type{}, D);
    step(I1{}, std::true_type{}, D);
  }
  ring = DmaRing{wcur, acur};
  __builtin_amdgcn_sched_barrier(0);  // (nothing that reads an accumulator may be scheduled above the wait states)
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last MFMAs have written their accumulators
  // The MFMAs are opaque to the compiler, which therefore adds no wait states of its own, and neither the memory
  // clobber nor the scheduling barrier orders a register-only accumulator read (v_accvgpr_read, an accumulator
  // spill) against the statement above: such reads were seen hoisted above it.  An empty statement that "modifies"
  // every accumulator after the wait states makes each later read depend on a point behind them.
#pragma unroll
  for (int ni = 0; ni < 8; ++ni)
#pragma unroll
    for (int j = 0; j < NJ; ++j) asm volatile("" : "+a"(acc[ni][j]));
  __builtin_amdgcn_sched_barrier(0);
  before_epilogue();

  // The store addresses are formed here, from lane indices that the compiler cannot trace back across the
  // K loop: computed ahead of it they were spilled, and every row of the epilogue began with a reload from
  // scratch memory (13 us per tile, with one wave per SIMD to hide it).
  int l16e = l16, kqe = kq;
  asm volatile("" : "+v"(l16e), "+v"(kqe));
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int m = (2 * j + wm) * 16 + l16e;
    if (m < cur.rows_left) {
#pragma unroll
      for (int ni = 0; ni < 8; ++ni) {
        const int n = cur.n_base + wn * 128 + ni * 16 + kqe * 4;  // a lane holds rows 4*(l/16)..+3 of the 16x16 tile D[n][m]
        store_quad<EPI, false>(Cout, aux, cur.crow0 + m, ldc, n, acc[ni][j][0], acc[ni][j][1], acc[ni][j][2], acc[ni][j][3]);
      }
    }
  }
}

// every variant executes the same loads and barriers; a wave row without live subtiles runs the
// one-subtile variant on clamped rows and stores nothing
template <int EPI, class F>
__device__ __forceinline__ void dma_tile_any(const DmaTile& cur, const DmaTile& nxt, const DmaLane& ln, DmaRing& ring,
                                             uint16_t* __restrict__ Cout, uint16_t* aux, uint32_t lds0, int KD, int lane, int wave,
                                             int ldc, F&& before_epilogue) {
  const int wm = wave >> 1, wn = wave & 1;
  const int nsub = min(16, (cur.rows_left + 15) >> 4);  // live 16-row subtiles of this tile
  const int nj = __builtin_amdgcn_readfirstlane((nsub - wm + 1) >> 1);  // ... of which this wave row owns nj (subtiles wm, wm+2, ...)
#define LOCMOE_DMA_TILE(N) dma_tile<N, EPI>(cur, nxt, ln, ring, Cout, aux, lds0, KD, wm, wn, lane, wave, ldc, before_epilogue)
  switch (nj) {
    case 8: LOCMOE_DMA_TILE(8); break;
    case 7: LOCMOE_DMA_TILE(7); break;
    case 6: LOCMOE_DMA_TILE(6); break;
    case 5: LOCMOE_DMA_TILE(5); break;
    case 4: LOCMOE_DMA_TILE(4); break;
    case 3: LOCMOE_DMA_TILE(3); break;
    case 2: LOCMOE_DMA_TILE(2); break;
    default: LOCMOE_DMA_TILE(1); break;
  }
#undef LOCMOE_DMA_TILE
}

// One tile per work-group, segments in buffer order: the shape of the grid for expert counts that the
// persistent kernel below does not take.
template <int EPI>
__global__ __launch_bounds__(kDmaThreads) void ffn_gemm_dma(const uint16_t* __restrict__ A,
                                                            const uint16_t* __restrict__ Wp,
                                                            uint16_t* __restrict__ Cout, uint16_t* aux,
                                                            const int32_t* __restrict__ seg_off,
                                                            const int32_t* __restrict__ buf_expert, int Kdim,
                                                            int Ndim, int MT, int NT) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tpe = MT * NT;
  const int within = blockIdx.x % tpe, r = blockIdx.x / tpe;
  const int mt = within % MT, nt = within / MT;
  const int seg0 = seg_off[r], rows = seg_off[r + 1] - seg0;
  if (mt * kBM >= rows) return;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const int KD = Kdim / (2 * kDmaBK);  // double steps
  const DmaTile cur = make_tile(A, Wp, seg0, rows, kBM, mt, nt, buf_expert[r], Kdim, Ndim);
  const DmaTile nxt = tail_alias(cur, KD);
  const DmaLane ln = make_lane(Kdim, wave, lane);
  DmaRing ring;
  dma_prefill(cur, ln, ring, lds0, wave, lane);
  dma_tile_any<EPI>(cur, nxt, ln, ring, Cout, aux, lds0, KD, lane, wave, Ndim, [] {});
  wait_vmcnt<0>();  // the tail prefetches must land before the LDS allocation is released
}

// Tile queues of the persistent kernel: 9 words of caller memory per launch.  Words 0..7 are the XCDs' next
// queue positions, word 8 counts the work-groups that are done with the queues.  All zero between launches:
// the caller hands them over zeroed once, and the last work-group of every launch puts them back.  The library
// keeps no queue of its own: entry points without a workspace argument run the same kernel with a fixed
// round-robin assignment of tiles instead (no claims, no state).
constexpr int kQueueWords = 16;  // one 64-byte set per launch

// A work-group is done with the queues (its last claim has returned); the last one of the grid clears them.
__device__ __forceinline__ void leave_queues(unsigned int* queue, unsigned groups) {
  __threadfence();
  if (atomicAdd(&queue[8], 1u) == groups - 1u) {
#pragma unroll
    for (int i = 0; i < 9; ++i) atomicExch(&queue[i], 0u);
  }
}

// Persistent form: one work-group per compute unit works through a queue of tiles, and the operand
// stream never drains between tiles: the last k-steps of a tile prefetch the first of the next, whose
// latency is hidden behind the epilogue.  With one work-group per tile every tile paid the launch of a
// 512-thread, 160 KiB group, the ordering preamble and a cold pipeline; for segments of at most 256 rows
// (no second m-tile to share the weight stream with) that was a third of the time.
//
// Which tiles.  Work-groups with ids congruent mod 8 run on one XCD (one L2).  The segments, ranked by
// descending row count, are dealt to the XCDs eight at a time in alternating direction; an XCD queues the
// tiles of its segments largest segment first; only non-empty tiles are enumerated, all tiles of a segment together with the m-tiles that share
// a weight tile adjacent.  The XCD's gridDim/8 work-groups start on the first gridDim/8 tiles and claim
// further ones from the queue (one atomic add per tile, issued before the epilogue and consumed after it,
// one tile ahead of the one being computed),
// so work-groups that run side by side hold neighbouring tiles (shared weight tile in L2), uneven tiles
// balance themselves, and the short tiles of ragged segments come last.  Every wave keeps the XCD's
// segment list in two registers (lane k: segment of local rank k and the inclusive tile count up to it;
// E/8 <= 64), built once in LDS before the pipeline starts.  The claimed index reaches the other waves
// through the one weight slot that is free between two tiles.
template <int EPI>
__global__ __launch_bounds__(kDmaThreads) void ffn_gemm_dma_persistent(const uint16_t* __restrict__ A,
                                                                       const uint16_t* __restrict__ Wp,
                                                                       uint16_t* __restrict__ Cout, uint16_t* aux,
                                                                       const int32_t* __restrict__ seg_off,
                                                                       const int32_t* __restrict__ buf_expert,
                                                                       int Kdim, int Ndim, int NT, int E,
                                                                       unsigned int* queue) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int xcd = blockIdx.x & 7, lb = blockIdx.x >> 3, stride = gridDim.x >> 3;
  const int nloc = E >> 3;  // segments of this XCD
  int32_t* s_seg = (int32_t*)smem;   // [E+1]
  int32_t* s_tab = s_seg + E + 1;    // [E/8]: segment of local rank k
  for (int t = tid; t <= E; t += kDmaThreads) s_seg[t] = seg_off[t];
  __syncthreads();
  for (int t = tid; t < E; t += kDmaThreads) {
    const int mine = s_seg[t + 1] - s_seg[t];
    int rank = 0;
    for (int q = 0; q < E; ++q) {
      const int other = s_seg[q + 1] - s_seg[q];
      rank += (other > mine || (other == mine && q < t)) ? 1 : 0;
    }
    // dealt in boustrophedon order (ranks 0..7 to XCDs 0..7, ranks 8..15 to XCDs 7..0, ...): every XCD gets
    // nearly the same number of rows; plain rank mod 8 always hands XCD 0 the largest of eight (+5 % rows on
    // the headline input, 1.3 % of the step's time)
    if ((((rank >> 3) & 1) ? 7 - (rank & 7) : (rank & 7)) == xcd) s_tab[rank >> 3] = t;
  }
  __syncthreads();
  int tab_seg = 0, tab_cum = 0;  // lane k < nloc: segment of local rank k, tiles of local ranks 0..k
  int tab_rows = 0;
  if (lane < nloc) {
    tab_seg = s_tab[lane];
    tab_rows = s_seg[tab_seg + 1] - s_seg[tab_seg];
  }
  auto count_tiles = [&](int bm) {  // fills tab_cum for m-tiles of at most bm rows, returns the XCD's tile count
    tab_cum = ((tab_rows + bm - 1) / bm) * NT;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(tab_cum, o, 64);
      if (lane >= o) tab_cum += up;
    }
    return __builtin_amdgcn_readfirstlane(__shfl(tab_cum, 63, 64));  // lanes past nloc carry the total
  };
  // m-tiles hold at most kBM rows, unless that leaves work-groups of this XCD without a tile (a short tile list:
  // few experts, narrow outputs): then at most kBM / 2 or kBM / 4 rows, two or four times as many tiles.  A short
  // tile costs most of a full one (the weight stream is the same), so this pays only for work-groups that would
  // idle otherwise.  Every output element is still summed by one lane in the same order: same bits.
  int bm = kBM;
  int total = count_tiles(bm);
  if (total > 0 && 2 * total <= stride) {
    bm = 4 * total <= stride ? kBM / 4 : kBM / 2;
    total = count_tiles(bm);
  }
  __syncthreads();  // everybody has read the tables before the pipeline overwrites this memory
  const bool multi = stride < total;     // else every tile of this XCD is somebody's first
  const bool dynamic = multi && queue;   // tiles beyond the first are claimed from the queue, else taken round-robin
  if (lb >= total) {
    if (queue && tid == 0) leave_queues(queue, gridDim.x);
    return;
  }

  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const int KD = Kdim / (2 * kDmaBK);  // double steps
  auto tile_at = [&](int jl) {
    const int k = __builtin_popcountll(__ballot(tab_cum <= jl));  // local rank of the segment that holds tile jl
    const int r = __builtin_amdgcn_readfirstlane(__shfl(tab_seg, k, 64));
    const int before = k ? __builtin_amdgcn_readfirstlane(__shfl(tab_cum, k - 1, 64)) : 0;
    const int within = jl - before;
    const int seg0 = seg_off[r], rows = seg_off[r + 1] - seg0;
    // A segment's rows are spread evenly over its m-tiles (in whole 16-row subtiles): m-tiles of one weight
    // tile that take equally long stay in step and share the weight stream through L2.  Cut at 256 rows, a
    // short last tile ran ahead of its partner, the stream was fetched twice and the kernel became HBM-bound
    // (272 rows per expert: 3.3 -> 2.45 ms for the second GEMM).
    const int mtc = (rows + bm - 1) / bm;
    const int span = ((rows + mtc - 1) / mtc + 15) & ~15;
    return make_tile(A, Wp, seg0, rows, span, within % mtc, within / mtc, buf_expert[r], Kdim, Ndim);
  };
  // `claimed`: the next tile of this work-group is number stride + claimed of the XCD's list
  int claimed = lb;
  if (dynamic && tid == 0) claimed = (int)atomicAdd(&queue[xcd], 1u);  // the tile after the first
  DmaTile cur = tile_at(lb);
  const DmaLane ln = make_lane(Kdim, wave, lane);
  DmaRing ring;
  dma_prefill(cur, ln, ring, lds0, wave, lane);
  for (;;) {
    // the claim goes from thread 0 to everybody through the one weight slot that is free between two tiles
    // (the tile's first k-step refills it: hence the second barrier)
    const int wfree = ring.wcur + 2 >= kWSlots ? ring.wcur + 2 - kWSlots : ring.wcur + 2;
    volatile int* mailbox = (volatile int*)(smem + kWRing + wfree * kWSlotBytes);
    if (tid == 0) *mailbox = claimed;
    __syncthreads();
    const int jn = multi ? stride + __builtin_amdgcn_readfirstlane(*mailbox) : total;
    __syncthreads();
    const bool more = jn < total;
    const DmaTile nxt = more ? tile_at(jn) : tail_alias(cur, KD);
    dma_tile_any<EPI>(cur, nxt, ln, ring, Cout, aux, lds0, KD, lane, wave, Ndim, [&] {
      if (more && tid == 0) claimed = dynamic ? (int)atomicAdd(&queue[xcd], 1u) : jn;
    });
    wait_vmcnt<0>();  // this tile's stores and the prefetches for the next (or the tail's) have all retired
    if (!more) break;
    cur = nxt;
  }
  if (queue && tid == 0) leave_queues(queue, gridDim.x);
}

// Weight packing (one-time): block (e, nt, kt) of 16 KiB is the LDS image of W[e][nt*256 .. +256][kt*32 .. +32]:
// 16-byte chunk p of the block holds row p/4, k-chunk (p%4) ^ (row/2 mod 4).
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint4* __restrict__ W, uint4* __restrict__ Wp,
                                                           int Ndim, int Kdim, long long chunks) {
  const long long q = (long long)blockIdx.x * 256 + threadIdx.x;
  if (q >= chunks) return;
  const int KT = Kdim / kDmaBK, NT = Ndim / kBN;
  const int p = (int)(q & 1023);
  long long blk = q >> 10;
  const int kt = (int)(blk % KT); blk /= KT;
  const int nt = (int)(blk % NT);
  const long long e = blk / NT;
  const int row = p >> 2, kc = (p & 3) ^ ((row >> 1) & 3);
  const long long src = ((e * Ndim + (long long)nt * kBN + row) * Kdim + (long long)kt * kDmaBK + kc * 8) / 8;
  Wp[q] = W[src];
}

// The packed layout of W^T straight from the row-major W [Rk rows, Cn columns] (the data gradients contract
// with the transposes): block (e, nt, kt) is the LDS image of W^T[nt*256 .. +256][kt*32 .. +32], i.e. of the
// 32 x 256 piece W[kt*32 ..][nt*256 ..].  The piece goes through LDS (512-byte rows, chunk index XORed with a
// 3-bit function of the row) and comes back through gfx950's transposing LDS read: 16 lanes receive the 8
// k-values of 16 consecutive columns, which is one 16-byte chunk of the packed block per lane.
typedef __attribute__((ext_vector_type(4))) short pk_s16x4;
__global__ __launch_bounds__(256) void transpose_pack_kernel(const uint16_t* __restrict__ W, uint4* __restrict__ Xp,
                                                             int Rk, int Cn) {
  __shared__ __attribute__((aligned(16))) char tile[32 * 512];
  const int KT = Rk / kDmaBK, NT = Cn / kBN;
  int blk = blockIdx.x;
  const int kt = blk % KT; blk /= KT;
  const int nt = blk % NT;
  const int e = blk / NT;
  const int t = threadIdx.x;
  const uint16_t* src = W + ((size_t)e * Rk + (size_t)kt * kDmaBK) * Cn + (size_t)nt * kBN;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = t + 256 * i, r = c >> 5, cc = c & 31;
    const uint4 v = *(const uint4*)(src + (size_t)r * Cn + cc * 8);
    const int sw = (r & 3) | (((r >> 3) & 1) << 2);
    *(uint4*)(tile + r * 512 + ((cc ^ (sw << 1)) << 4)) = v;
  }
  __syncthreads();
  const int lane = t & 63, wave = t >> 6, g = lane >> 4, s16 = lane & 15;
  const int sw = (s16 >> 2) | ((g & 1) << 2);
  const int row = 8 * g + (s16 >> 2), b1 = (s16 & 3) >> 1, inner = (s16 & 1) * 8;
  uint4* dst = Xp + (size_t)blockIdx.x * 1024;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int nbase = 16 * (wave + 4 * it);
    const char* p = tile + row * 512 + ((((nbase >> 3) + b1) ^ (sw << 1)) << 4) + inner;
    const pk_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pk_s16x4 __attribute__((address_space(3)))*)p);
    const pk_s16x4 hi =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((pk_s16x4 __attribute__((address_space(3)))*)(p + 4 * 512));
    // this lane now holds W^T[n][8 g .. 8 g + 7] for n = nbase + s16: k-chunk g of packed row n
    const int n = nbase + s16;
    uint4 v;
    v.x = (uint32_t)(uint16_t)lo[0] | ((uint32_t)(uint16_t)lo[1] << 16);
    v.y = (uint32_t)(uint16_t)lo[2] | ((uint32_t)(uint16_t)lo[3] << 16);
    v.z = (uint32_t)(uint16_t)hi[0] | ((uint32_t)(uint16_t)hi[1] << 16);
    v.w = (uint32_t)(uint16_t)hi[2] | ((uint32_t)(uint16_t)hi[3] << 16);
    dst[n * 4 + (g ^ ((n >> 1) & 3))] = v;
  }
}

template <int EPI>
int launch_dma(const void* A, const void* Wp, void* C, void* aux, const int32_t* seg_off, const int32_t* buf_expert, int E,
               int rows_max, int Kdim, int Ndim, unsigned int* queue, hipStream_t st) {
  const int MT = ceil_div(rows_max, kBM), NT = Ndim / kBN;
  const long long total = (long long)E * MT * NT;
  if (total > 0x7FFFFFFFLL) return LOCMOE_ERR_SHAPE;
  static std::atomic<uint64_t> lds_allowed[2];  // per kernel of this instantiation: devices whose LDS limit is raised
  if (E % 8 == 0 && E <= 512) {
    auto kern = ffn_gemm_dma_persistent<EPI>;
    if (!allow_lds((const void*)kern, kDmaSmem, lds_allowed[0])) return LOCMOE_ERR_HIP;
    // one work-group per compute unit (160 KiB of LDS each), a multiple of 8 so that every XCD gets as many
    // (up to four work-groups per tile of the upper bound: the kernel cuts the m-tiles of a short list finer)
    const long long groups = std::min<long long>((cu_count() / 8) * 8, (4 * total + 7) / 8 * 8);
    hipLaunchKernelGGL(kern, dim3((unsigned)groups), dim3(kDmaThreads), kDmaSmem, st, (const uint16_t*)A,
                       (const uint16_t*)Wp, (uint16_t*)C, (uint16_t*)aux, seg_off, buf_expert, Kdim, Ndim, NT, E, queue);
    return launch_status();
  }
  auto kern = ffn_gemm_dma<EPI>;
  if (!allow_lds((const void*)kern, kDmaSmem, lds_allowed[1])) return LOCMOE_ERR_HIP;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(kDmaThreads), kDmaSmem, st, (const uint16_t*)A,
                     (const uint16_t*)Wp, (uint16_t*)C, (uint16_t*)aux, seg_off, buf_expert, Kdim, Ndim, MT, NT);
  return launch_status();
}

// out[z][c][r] = in[z][r][c] for bf16 matrices whose sides are multiples of 8: 64x64 tiles through LDS,
// 16-byte global accesses on both sides.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ in,
                                                             uint16_t* __restrict__ out, int R, int Cc) {
  __shared__ uint16_t tile[64][66];  // 33 words per row: the column reads below fall into distinct banks
  const size_t base = (size_t)blockIdx.z * R * Cc;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int t = threadIdx.x, ch = t & 7;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int row = (t >> 3) + 32 * k;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r0 + row < R && c0 + ch * 8 < Cc) v = *(const uint4*)(in + base + (size_t)(r0 + row) * Cc + c0 + ch * 8);
    uint32_t* dst = (uint32_t*)&tile[row][ch * 8];
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int col = (t >> 3) + 32 * k;  // a column of the input tile = a row of the output
    if (c0 + col < Cc && r0 + ch * 8 < R) {
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        w[i] = (uint32_t)tile[ch * 8 + 2 * i][col] | ((uint32_t)tile[ch * 8 + 2 * i + 1][col] << 16);
      *(uint4*)(out + base + (size_t)(c0 + col) * R + r0 + ch * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

// shapes the packed layout and the DMA kernel support
inline bool packable(const locmoe_desc* p) {
  return p->d % kBN == 0 && p->h % kBN == 0 && (long long)p->d * 2 * 256 < 0x7FFFFFFFLL &&
         (long long)p->h * 2 * 256 < 0x7FFFFFFFLL;
}

template <bool A_F32, int EPI, bool OUT_F32>
int launch_gemm(const void* A, const void* W, void* C, void* aux, const int32_t* seg_off, const int32_t* buf_expert, int E,
                int rows_max, int Kdim, int Ndim, hipStream_t st) {
  if (!A_F32 && Kdim % kBK == 0 && Ndim % kBN == 0) {
    const int MT = ceil_div(rows_max, kBM), NT = Ndim / kBN;
    const long long total = (long long)E * MT * NT;
    if (total <= 0x7FFFFFFFLL) {
      auto kern = ffn_gemm_256<EPI, OUT_F32, 1>;
      static std::atomic<uint64_t> lds_allowed;
      if (!allow_lds((const void*)kern, kFastSmem, lds_allowed)) return LOCMOE_ERR_HIP;
      hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(kFastThreads), kFastSmem, st, (const uint16_t*)A,
                         (const uint16_t*)W, C, (uint16_t*)aux, seg_off, buf_expert, Kdim, Ndim, MT, NT, (int)total);
      return launch_status();
    }
  }
  const int MT = ceil_div(rows_max, 64);
  if ((long long)E * MT > 65535) return LOCMOE_ERR_SHAPE;
  hipLaunchKernelGGL((ffn_gemm_generic<A_F32, EPI, OUT_F32>), dim3(ceil_div(Ndim, 64), E * MT),
                     dim3(kGenThreads), 0, st, A, (const uint16_t*)W, C, (uint16_t*)aux, seg_off, buf_expert, Kdim, Ndim, MT);
  return launch_status();
}

}  // namespace
}  // namespace locmoe

namespace locmoe {
namespace {

// C[rows, h] = epilogue(A[rows, d] . W[h, d]^T): the first GEMM of Eq. 1 and, with the transposed W_out in
// place of W_in, the first GEMM of its backward.  `queue`: 9 zeroed words of caller memory for the tile claims of
// the packed-weight kernel, or nullptr (fixed tile assignment).
template <int EPI>
int gemm_d_to_h(const locmoe_desc* desc, const void* A, const int32_t* seg_off, const int32_t* buf_expert,
                const void* W, void* Cbf16, void* aux, unsigned int* queue, void* stream) {
  const int rows_max = desc->C < desc->T ? desc->C : desc->T;  // kept[e] <= min(C, T)
  if (desc->w_packed) {
    if (desc->x_dtype != LOCMOE_BF16 || !packable(desc)) return LOCMOE_ERR_ARG;
    return launch_dma<EPI>(A, W, Cbf16, aux, seg_off, buf_expert, desc->E, rows_max, desc->d, desc->h, queue,
                           as_stream(stream));
  }
  if (desc->x_dtype == LOCMOE_F32)
    return launch_gemm<true, EPI, false>(A, W, Cbf16, aux, seg_off, buf_expert, desc->E, rows_max, desc->d, desc->h,
                                         as_stream(stream));
  return launch_gemm<false, EPI, false>(A, W, Cbf16, aux, seg_off, buf_expert, desc->E, rows_max, desc->d, desc->h,
                                        as_stream(stream));
}

// C[rows, d] = A[rows, h] . W[d, h]^T, A bf16, C of the storage type: the second GEMM of Eq. 1 and, with the
// transposed W_in in place of W_out, the second GEMM of its backward
int gemm_h_to_d(const locmoe_desc* desc, const void* A, const int32_t* seg_off, const int32_t* buf_expert,
                const void* W, void* C, unsigned int* queue, void* stream) {
  const int rows_max = desc->C < desc->T ? desc->C : desc->T;
  if (desc->w_packed) {
    if (desc->x_dtype != LOCMOE_BF16 || !packable(desc)) return LOCMOE_ERR_ARG;
    return launch_dma<kEpiNone>(A, W, C, nullptr, seg_off, buf_expert, desc->E, rows_max, desc->h, desc->d, queue,
                                as_stream(stream));
  }
  if (desc->x_dtype == LOCMOE_F32)
    return launch_gemm<false, kEpiNone, true>(A, W, C, nullptr, seg_off, buf_expert, desc->E, rows_max, desc->h,
                                              desc->d, as_stream(stream));
  return launch_gemm<false, kEpiNone, false>(A, W, C, nullptr, seg_off, buf_expert, desc->E, rows_max, desc->h,
                                             desc->d, as_stream(stream));
}

// The two queue sets of a workspace (first and second GEMM of a call); nullptr when the caller gave none.
inline unsigned int* queue_set(void* ws, int which) {
  return ws ? (unsigned int*)ws + which * kQueueWords : nullptr;
}
inline bool ws_ok(const void* ws, size_t ws_bytes) {
  return ws && ws_bytes >= LOCMOE_FFN_WS_BYTES && ((uintptr_t)ws & 3u) == 0;
}

int ffn_in(const locmoe_desc* desc, const void* send, const int32_t* seg_off, const int32_t* buf_expert,
           const void* W_in, void* H_ws, void* Z, void* ws, void* stream) {
  if (!desc || !send || !seg_off || !buf_expert || !W_in || !H_ws) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  if (Z) return gemm_d_to_h<kEpiGeluSave>(desc, send, seg_off, buf_expert, W_in, H_ws, Z, queue_set(ws, 0), stream);
  return gemm_d_to_h<kEpiGelu>(desc, send, seg_off, buf_expert, W_in, H_ws, nullptr, queue_set(ws, 0), stream);
}

int ffn_out(const locmoe_desc* desc, const void* H_ws, const int32_t* seg_off, const int32_t* buf_expert,
            const void* W_out, void* out, void* ws, void* stream) {
  if (!desc || !H_ws || !seg_off || !buf_expert || !W_out || !out) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  return gemm_h_to_d(desc, H_ws, seg_off, buf_expert, W_out, out, queue_set(ws, 1), stream);
}

int ffn_dgrad(const locmoe_desc* desc, const void* dout, const void* Z, const int32_t* seg_off,
              const int32_t* buf_expert, const void* W_out_t, const void* W_in_t, void* dZ, void* dsend, void* ws,
              void* stream) {
  if (!desc || !dout || !Z || !seg_off || !buf_expert || !W_out_t || !W_in_t || !dZ || !dsend) return LOCMOE_ERR_NULL;
  int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  // dZ = (dout . W_out) * GeLU'(Z): W_out^T is [h,d], the orientation of W_in
  st = gemm_d_to_h<kEpiGeluGrad>(desc, dout, seg_off, buf_expert, W_out_t, dZ, const_cast<void*>(Z), queue_set(ws, 0),
                                 stream);
  if (st != LOCMOE_OK) return st;
  // dsend = dZ . W_in: W_in^T is [d,h], the orientation of W_out
  return gemm_h_to_d(desc, dZ, seg_off, buf_expert, W_in_t, dsend, queue_set(ws, 1), stream);
}

}  // namespace
}  // namespace locmoe

using namespace locmoe;

// ---- without a workspace: stateless, fixed tile assignment ---------------------------------------------------
extern "C" int locmoe_expert_ffn_in(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                    const int32_t* buf_expert, const void* W_in, void* H_ws, void* stream) {
  return ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, nullptr, nullptr, stream);
}

extern "C" int locmoe_expert_ffn_in_save(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                         const int32_t* buf_expert, const void* W_in, void* H_ws, void* Z,
                                         void* stream) {
  if (!Z) return LOCMOE_ERR_NULL;
  return ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, Z, nullptr, stream);
}

extern "C" int locmoe_expert_ffn_out(const locmoe_desc* desc, const void* H_ws, const int32_t* seg_off,
                                     const int32_t* buf_expert, const void* W_out, void* out, void* stream) {
  return ffn_out(desc, H_ws, seg_off, buf_expert, W_out, out, nullptr, stream);
}

extern "C" int locmoe_expert_ffn_dgrad(const locmoe_desc* desc, const void* dout, const void* Z,
                                       const int32_t* seg_off, const int32_t* buf_expert, const void* W_out_t,
                                       const void* W_in_t, void* dZ, void* dsend, void* stream) {
  return ffn_dgrad(desc, dout, Z, seg_off, buf_expert, W_out_t, W_in_t, dZ, dsend, nullptr, stream);
}

extern "C" int locmoe_expert_ffn(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                 const int32_t* buf_expert, const void* W_in, const void* W_out, void* H_ws,
                                 void* out, void* stream) {
  if (!W_out || !out) return LOCMOE_ERR_NULL;
  const int st = ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, nullptr, nullptr, stream);
  if (st != LOCMOE_OK) return st;
  return ffn_out(desc, H_ws, seg_off, buf_expert, W_out, out, nullptr, stream);
}

// ---- with a caller workspace: the packed-weight kernels claim their tiles from it -----------------------------
extern "C" int locmoe_expert_ffn_in_ws(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                       const int32_t* buf_expert, const void* W_in, void* H_ws, void* ws,
                                       size_t ws_bytes, void* stream) {
  if (!ws_ok(ws, ws_bytes)) return LOCMOE_ERR_WORKSPACE;
  return ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, nullptr, ws, stream);
}

extern "C" int locmoe_expert_ffn_in_save_ws(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                            const int32_t* buf_expert, const void* W_in, void* H_ws, void* Z, void* ws,
                                            size_t ws_bytes, void* stream) {
  if (!Z) return LOCMOE_ERR_NULL;
  if (!ws_ok(ws, ws_bytes)) return LOCMOE_ERR_WORKSPACE;
  return ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, Z, ws, stream);
}

extern "C" int locmoe_expert_ffn_out_ws(const locmoe_desc* desc, const void* H_ws, const int32_t* seg_off,
                                        const int32_t* buf_expert, const void* W_out, void* out, void* ws,
                                        size_t ws_bytes, void* stream) {
  if (!ws_ok(ws, ws_bytes)) return LOCMOE_ERR_WORKSPACE;
  return ffn_out(desc, H_ws, seg_off, buf_expert, W_out, out, ws, stream);
}

extern "C" int locmoe_expert_ffn_dgrad_ws(const locmoe_desc* desc, const void* dout, const void* Z,
                                          const int32_t* seg_off, const int32_t* buf_expert, const void* W_out_t,
                                          const void* W_in_t, void* dZ, void* dsend, void* ws, size_t ws_bytes,
                                          void* stream) {
  if (!ws_ok(ws, ws_bytes)) return LOCMOE_ERR_WORKSPACE;
  return ffn_dgrad(desc, dout, Z, seg_off, buf_expert, W_out_t, W_in_t, dZ, dsend, ws, stream);
}

extern "C" int locmoe_expert_ffn_ws(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                    const int32_t* buf_expert, const void* W_in, const void* W_out, void* H_ws,
                                    void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!W_out || !out) return LOCMOE_ERR_NULL;
  if (!ws_ok(ws, ws_bytes)) return LOCMOE_ERR_WORKSPACE;
  const int st = ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, nullptr, ws, stream);
  if (st != LOCMOE_OK) return st;
  return ffn_out(desc, H_ws, seg_off, buf_expert, W_out, out, ws, stream);
}

extern "C" int locmoe_transpose_weights(const locmoe_desc* desc, const void* W_in, const void* W_out, void* W_in_t,
                                        void* W_out_t, void* stream) {
  using namespace locmoe;
  if (!desc || !W_in || !W_out || !W_in_t || !W_out_t) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  const int tiles_h = ceil_div(desc->h, 64), tiles_d = ceil_div(desc->d, 64);
  if (tiles_h > 65535 || tiles_d > 65535 || desc->E > 65535) return LOCMOE_ERR_SHAPE;
  hipStream_t s = as_stream(stream);
  // W_in[e] is [h,d] -> [d,h];  W_out[e] is [d,h] -> [h,d]
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3(tiles_d, tiles_h, desc->E), dim3(256), 0, s, (const uint16_t*)W_in,
                     (uint16_t*)W_in_t, desc->h, desc->d);
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3(tiles_h, tiles_d, desc->E), dim3(256), 0, s, (const uint16_t*)W_out,
                     (uint16_t*)W_out_t, desc->d, desc->h);
  return launch_status();
}

extern "C" int locmoe_pack_weights_t(const locmoe_desc* desc, const void* W_in, const void* W_out,
                                     void* W_in_t_packed, void* W_out_t_packed, void* stream) {
  using namespace locmoe;
  if (!desc || !W_in || !W_out || !W_in_t_packed || !W_out_t_packed) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  if (!packable(desc)) return LOCMOE_ERR_SHAPE;
  const long long blocks = (long long)desc->E * (desc->h / kBN) * (desc->d / kDmaBK);  // = E (d/256) (h/32) as well
  if (blocks > 0x7FFFFFFFLL) return LOCMOE_ERR_SHAPE;
  hipStream_t s = as_stream(stream);
  // W_in[e] is [h,d]: its transpose has N = d rows and K = h;  W_out[e] is [d,h]: N = h, K = d
  hipLaunchKernelGGL(transpose_pack_kernel, dim3((unsigned)((long long)desc->E * (desc->d / kBN) * (desc->h / kDmaBK))),
                     dim3(256), 0, s, (const uint16_t*)W_in, (uint4*)W_in_t_packed, desc->h, desc->d);
  hipLaunchKernelGGL(transpose_pack_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const uint16_t*)W_out,
                     (uint4*)W_out_t_packed, desc->d, desc->h);
  return launch_status();
}

extern "C" size_t locmoe_packed_weights_bytes(const locmoe_desc* desc) {
  using namespace locmoe;
  if (check_desc(desc) != LOCMOE_OK || !packable(desc)) return 0;
  return (size_t)desc->E * (size_t)desc->h * (size_t)desc->d * 2;
}

extern "C" int locmoe_pack_weights(const locmoe_desc* desc, const void* W_in, const void* W_out, void* W_in_packed,
                                   void* W_out_packed, void* stream) {
  using namespace locmoe;
  if (!desc || !W_in || !W_out || !W_in_packed || !W_out_packed) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  if (!packable(desc)) return LOCMOE_ERR_SHAPE;
  const long long chunks = (long long)desc->E * desc->h * desc->d / 8;
  const unsigned blocks = (unsigned)((chunks + 255) / 256);
  hipStream_t s = as_stream(stream);
  hipLaunchKernelGGL(pack_weights_kernel, dim3(blocks), dim3(256), 0, s, (const uint4*)W_in, (uint4*)W_in_packed,
                     desc->h, desc->d, chunks);  // W_in[e] is [h rows, d]: N = h, K = d
  hipLaunchKernelGGL(pack_weights_kernel, dim3(blocks), dim3(256), 0, s, (const uint4*)W_out, (uint4*)W_out_packed,
                     desc->d, desc->h, chunks);  // W_out[e] is [d rows, h]: N = d, K = h
  return launch_status();
}
