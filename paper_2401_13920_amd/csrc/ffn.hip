// Expert FFN of Eq. 1 as two grouped GEMMs over the send buffer's expert segments:
//   H = GeLU(S_e . W_in[e]^T)   (rows x h, rounded once to bf16)
//   O = H . W_out[e]^T          (rows x d, rounded once to the storage type)
// Both weights are stored row-major in Eq. 1's orientation ([h,d] and [d,h]), so both GEMMs
// contract over the contiguous axis of both operands ("NT" form): every MFMA fragment is one
// 16-byte LDS read.  bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// The weight rows feed the MFMA's A operand and the activation rows its B operand, i.e. the
// tile is computed transposed (D[n][m]); a lane then owns 4 consecutive output columns n of one
// row m per accumulator quad and stores them as one 8-byte (bf16) or 16-byte (fp32) vector.
#include <math.h>

#include "common.h"

namespace locmoe {
namespace {

__device__ __forceinline__ float gelu_erf(float v) {  // v * Phi(v)
  return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
}

__device__ __forceinline__ f32x16 mfma_bf16(const bf16x8& a, const bf16x8& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// One accumulator quad -> memory.  q holds D[n0..n0+3][m] for one row m.
template <bool GELU, bool OUT_F32>
__device__ __forceinline__ void store_quad(void* C, size_t row, int ldc, int n0, float q0, float q1, float q2,
                                           float q3) {
  if (GELU) { q0 = gelu_erf(q0); q1 = gelu_erf(q1); q2 = gelu_erf(q2); q3 = gelu_erf(q3); }
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

template <bool A_F32, bool GELU, bool OUT_F32>
__global__ __launch_bounds__(kGenThreads) void ffn_gemm_generic(const void* __restrict__ A,
                                                                const uint16_t* __restrict__ W,
                                                                void* __restrict__ Cout,
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
        store_quad<GELU, OUT_F32>(Cout, (size_t)seg0 + m, Ndim, n, acc[vq * 4 + 0], acc[vq * 4 + 1],
                                  acc[vq * 4 + 2], acc[vq * 4 + 3]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Tuned kernel: 256x256x64 tile, 8 waves (2 along m x 4 along n, 128x64 per wave), double
// buffered LDS (2 x 64 KiB), XOR-swizzled 16-byte slots, bf16 activations, K % 64 == 0,
// N % 256 == 0.  Work-group ids are remapped so that each XCD (ids congruent mod 8 land on one
// XCD and share its L2) walks a contiguous range of experts, with the m-tiles that share a
// weight tile adjacent in time.
// ---------------------------------------------------------------------------------------------
constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kFastThreads = 512;
constexpr int kStageBytes = (kBM + kBN) * kBK * 2;  // 64 KiB
constexpr int kFastSmem = 2 * kStageBytes;

template <int SH>
__device__ __forceinline__ int swz(int row, int chunk) { return (chunk ^ ((row >> SH) & 7)) << 4; }

template <bool GELU, bool OUT_F32, int SH>
__global__ __launch_bounds__(kFastThreads) void ffn_gemm_256(const uint16_t* __restrict__ A,
                                                             const uint16_t* __restrict__ W,
                                                             void* __restrict__ Cout,
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
          store_quad<GELU, OUT_F32>(Cout, (size_t)seg0 + m, Ndim, n, acc[ni][mi][vq * 4 + 0],
                                    acc[ni][mi][vq * 4 + 1], acc[ni][mi][vq * 4 + 2], acc[ni][mi][vq * 4 + 3]);
        }
    }
  }
}

template <bool A_F32, bool GELU, bool OUT_F32>
int launch_gemm(const void* A, const void* W, void* C, const int32_t* seg_off, const int32_t* buf_expert, int E,
                int rows_max, int Kdim, int Ndim, hipStream_t st) {
  if (!A_F32 && Kdim % kBK == 0 && Ndim % kBN == 0) {
    const int MT = ceil_div(rows_max, kBM), NT = Ndim / kBN;
    const long long total = (long long)E * MT * NT;
    if (total <= 0x7FFFFFFFLL) {
      auto kern = ffn_gemm_256<GELU, OUT_F32, 0>;
      if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kFastSmem) !=
          hipSuccess)
        return LOCMOE_ERR_HIP;
      hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(kFastThreads), kFastSmem, st, (const uint16_t*)A,
                         (const uint16_t*)W, C, seg_off, buf_expert, Kdim, Ndim, MT, NT, (int)total);
      return launch_status();
    }
  }
  const int MT = ceil_div(rows_max, 64);
  if ((long long)E * MT > 65535) return LOCMOE_ERR_SHAPE;
  hipLaunchKernelGGL((ffn_gemm_generic<A_F32, GELU, OUT_F32>), dim3(ceil_div(Ndim, 64), E * MT),
                     dim3(kGenThreads), 0, st, A, (const uint16_t*)W, C, seg_off, buf_expert, Kdim, Ndim, MT);
  return launch_status();
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_expert_ffn_in(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                    const int32_t* buf_expert, const void* W_in, void* H_ws, void* stream) {
  using namespace locmoe;
  if (!desc || !send || !seg_off || !buf_expert || !W_in || !H_ws) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  const int rows_max = desc->C < desc->T ? desc->C : desc->T;  // kept[e] <= min(C, T)
  if (desc->x_dtype == LOCMOE_F32)
    return launch_gemm<true, true, false>(send, W_in, H_ws, seg_off, buf_expert, desc->E, rows_max, desc->d,
                                          desc->h, as_stream(stream));
  return launch_gemm<false, true, false>(send, W_in, H_ws, seg_off, buf_expert, desc->E, rows_max, desc->d,
                                         desc->h, as_stream(stream));
}

extern "C" int locmoe_expert_ffn_out(const locmoe_desc* desc, const void* H_ws, const int32_t* seg_off,
                                     const int32_t* buf_expert, const void* W_out, void* out, void* stream) {
  using namespace locmoe;
  if (!desc || !H_ws || !seg_off || !buf_expert || !W_out || !out) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  const int rows_max = desc->C < desc->T ? desc->C : desc->T;
  if (desc->x_dtype == LOCMOE_F32)
    return launch_gemm<false, false, true>(H_ws, W_out, out, seg_off, buf_expert, desc->E, rows_max, desc->h,
                                           desc->d, as_stream(stream));
  return launch_gemm<false, false, false>(H_ws, W_out, out, seg_off, buf_expert, desc->E, rows_max, desc->h,
                                          desc->d, as_stream(stream));
}

extern "C" int locmoe_expert_ffn(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                 const int32_t* buf_expert, const void* W_in, const void* W_out, void* H_ws,
                                 void* out, void* stream) {
  if (!W_out || !out) return LOCMOE_ERR_NULL;
  const int st = locmoe_expert_ffn_in(desc, send, seg_off, buf_expert, W_in, H_ws, stream);
  if (st != LOCMOE_OK) return st;
  return locmoe_expert_ffn_out(desc, H_ws, seg_off, buf_expert, W_out, out, stream);
}
