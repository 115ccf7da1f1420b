// The routers the paper compares LocMoE with (Section 2, Section 4), as far as they differ from the LocMoE path:
//   - the gate as a dense layer with a learned weight (Section 3.2.1; the switch router's gate, which GrAP
//     replaces): g[m,i] = omega_i . x_m, a [T,d] x [d,E] contraction.  Top-1 selection, the score and the
//     auxiliary loss of Eq. 5 are locmoe_route's, unchanged.
//   - hash routing: the expert is a fixed, parameter-free function of the token's key; no token feature is read.
// Dispatch, expert FFN and combine are the same kernels for all three routers.
#include "common.h"

namespace locmoe {
namespace {

// ---------------------------------------------------------------------------------------------
// Dense gate, bf16 storage, d a multiple of 64: 128 tokens x up to 128 experts per work-group, four waves of
// 32 tokens each, v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  E is small, so the kernel is bound by the
// one pass over x (T d 2 bytes): 2 T d E flops are 64 flops per byte at E = 64, far below the machine's ridge.
// The weight [E,d] is re-read by every work-group from L2.  Operands go global -> registers -> LDS (16-byte
// chunks, chunk index XORed with row/2 so that a fragment read of 32 rows touches every bank equally); the next
// k-step's loads are in flight while the current one is multiplied.
// ---------------------------------------------------------------------------------------------
constexpr int kDgThreads = 256;
constexpr int kDgTokens = 128;                       // tokens per work-group
constexpr int kDgBK = 64;                            // k-step
constexpr int kDgRowBytes = kDgBK * 2;               // 128 B per LDS row
constexpr int kDgTile = 128 * kDgRowBytes;           // 16 KiB: 128 rows of one operand
constexpr int kDgSmem = 4 * kDgTile;                 // x and W, double buffered

__device__ __forceinline__ int dg_swz(int row, int chunk) { return (chunk ^ ((row >> 1) & 7)) << 4; }

template <int NT>  // 32-expert tiles per pass: experts [e0, e0 + 32 NT)
__global__ __launch_bounds__(kDgThreads) void gate_dense_mfma_kernel(const uint16_t* __restrict__ x,
                                                                     const uint16_t* __restrict__ Wg,
                                                                     float* __restrict__ g, int T, int d, int E) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = blockIdx.x * kDgTokens;
  const int e0 = blockIdx.y * 128;
  // global -> LDS assignment: four x chunks and NT W chunks of 16 bytes per thread and k-step
  const uint16_t* gx[4];
  const uint16_t* gw[NT];
  int lds_x[4], lds_w[NT];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + i * kDgThreads, row = c >> 3, kc = c & 7;
    gx[i] = x + (size_t)min(m0 + row, T - 1) * d + kc * 8;  // rows past T re-read the last token (never stored)
    lds_x[i] = row * kDgRowBytes + dg_swz(row, kc);
  }
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int c = tid + i * kDgThreads, row = c >> 3, kc = c & 7;
    gw[i] = Wg + (size_t)min(e0 + row, E - 1) * d + kc * 8;  // rows past E re-read the last expert (never stored)
    lds_w[i] = row * kDgRowBytes + dg_swz(row, kc);
  }
  const int frow = lane & 31, khalf = lane >> 5;
  const int xrow = wave * 32 + frow;

  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = (f32x16){0};

  u32x4 rx[4], rw[NT];
#pragma unroll
  for (int i = 0; i < 4; ++i) rx[i] = *(const u32x4*)gx[i];
#pragma unroll
  for (int i = 0; i < NT; ++i) rw[i] = *(const u32x4*)gw[i];
#pragma unroll
  for (int i = 0; i < 4; ++i) *(u32x4*)(smem + lds_x[i]) = rx[i];
#pragma unroll
  for (int i = 0; i < NT; ++i) *(u32x4*)(smem + 2 * kDgTile + lds_w[i]) = rw[i];
  __syncthreads();

  const int KT = d / kDgBK;
  for (int kt = 0; kt < KT; ++kt) {
    const int ko = min(kt + 1, KT - 1) * kDgBK;  // (the step after the last re-reads the last: never consumed)
#pragma unroll
    for (int i = 0; i < 4; ++i) rx[i] = *(const u32x4*)(gx[i] + ko);
#pragma unroll
    for (int i = 0; i < NT; ++i) rw[i] = *(const u32x4*)(gw[i] + ko);
    const char* sx = smem + (kt & 1) * kDgTile;
    const char* sw = smem + 2 * kDgTile + (kt & 1) * kDgTile;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int kc = ks * 2 + khalf;
      const bf16x8 fx = *(const bf16x8*)(sx + xrow * kDgRowBytes + dg_swz(xrow, kc));
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int wrow = t * 32 + frow;
        const bf16x8 fw = *(const bf16x8*)(sw + wrow * kDgRowBytes + dg_swz(wrow, kc));
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fx, acc[t], 0, 0, 0);  // D[expert][token]
      }
    }
    char* dx = smem + ((kt + 1) & 1) * kDgTile;
    char* dw = smem + 2 * kDgTile + ((kt + 1) & 1) * kDgTile;
#pragma unroll
    for (int i = 0; i < 4; ++i) *(u32x4*)(dx + lds_x[i]) = rx[i];
#pragma unroll
    for (int i = 0; i < NT; ++i) *(u32x4*)(dw + lds_w[i]) = rw[i];
    __syncthreads();
  }
  // a lane holds experts e0 + 32 t + 8 vq + 4 khalf .. +3 of token m0 + 32 wave + frow
  const int m = m0 + xrow;
  if (m < T) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int i0 = e0 + t * 32 + vq * 8 + khalf * 4;
        float* dst = g + (size_t)m * E + i0;
        if (i0 + 3 < E && (E & 3) == 0) {
          *(float4*)dst = make_float4(acc[t][vq * 4 + 0], acc[t][vq * 4 + 1], acc[t][vq * 4 + 2], acc[t][vq * 4 + 3]);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (i0 + q < E) dst[q] = acc[t][vq * 4 + q];
        }
      }
  }
}

// Any shape and either storage type: one wave per token, lanes stride over the features, the wave's sum by a
// fixed butterfly.  Correct for every descriptor; used for fp32 storage and hidden sizes that are no multiple of 64.
template <bool BF16>
__global__ __launch_bounds__(256) void gate_dense_generic_kernel(const void* __restrict__ x,
                                                                 const void* __restrict__ Wg,
                                                                 float* __restrict__ g, int T, int d, int E) {
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (m >= T) return;
  for (int i = 0; i < E; ++i) {
    float s = 0.f;
    for (int j = lane; j < d; j += kWave) {
      float a, b;
      if (BF16) {
        a = bf16_bits_to_f32(((const uint16_t*)x)[(size_t)m * d + j]);
        b = bf16_bits_to_f32(((const uint16_t*)Wg)[(size_t)i * d + j]);
      } else {
        a = ((const float*)x)[(size_t)m * d + j];
        b = ((const float*)Wg)[(size_t)i * d + j];
      }
      s = fmaf(a, b, s);
    }
    s = group_sum<kWave>(s);
    if (lane == 0) g[(size_t)m * E + i] = s;
  }
}

// ---------------------------------------------------------------------------------------------
// Hash routing.  The 32-bit finalizer of MurmurHash3 (a published bijective mixer of 32-bit integers):
// xor-shift 16, times 0x85EBCA6B, xor-shift 13, times 0xC2B2AE35, xor-shift 16.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t mix32(uint32_t v) {
  v ^= v >> 16;
  v *= 0x85EBCA6Bu;
  v ^= v >> 13;
  v *= 0xC2B2AE35u;
  v ^= v >> 16;
  return v;
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

constexpr int kHashThreads = 256, kHashPerThread = 8;

// eid, w and the per-expert counts.  Counts: LDS histogram per block, one integer atomic per non-empty cell
// into cnt (integer sums: the result does not depend on the order).
__global__ __launch_bounds__(kHashThreads) void route_hash_kernel(const int32_t* __restrict__ key, uint32_t offset,
                                                                  int32_t* __restrict__ eid, float* __restrict__ w,
                                                                  int32_t* __restrict__ cnt, int T, int E) {
  extern __shared__ int32_t hist[];
  for (int i = threadIdx.x; i < E; i += kHashThreads) hist[i] = 0;
  __syncthreads();
  const int base = blockIdx.x * kHashThreads * kHashPerThread;
#pragma unroll
  for (int k = 0; k < kHashPerThread; ++k) {
    const int m = base + k * kHashThreads + threadIdx.x;
    if (m < T) {
      const uint32_t kv = key ? (uint32_t)key[m] : (uint32_t)m;
      const int e = (int)(mix32(kv + offset) % (uint32_t)E);
      eid[m] = e;
      w[m] = 1.0f;
      atomicAdd(&hist[e], 1);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < E; i += kHashThreads)
    if (hist[i]) atomicAdd(&cnt[i], hist[i]);
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_gate_dense(const locmoe_desc* desc, const void* x, const void* Wg, float* g, void* stream) {
  using namespace locmoe;
  if (!desc || !x || !Wg || !g) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  hipStream_t s = as_stream(stream);
  const int T = desc->T, d = desc->d, E = desc->E;
  if (desc->x_dtype == LOCMOE_BF16 && d % kDgBK == 0) {
    const int passes = ceil_div(E, 128);
    const int nt = passes > 1 ? 4 : ceil_div(E, 32);  // 32-expert tiles per pass
    const dim3 grid(ceil_div(T, kDgTokens), passes);
#define LOCMOE_DG(N)                                                                                             \
  {                                                                                                              \
    static std::atomic<uint64_t> lds_allowed;                                                                    \
    auto kern = gate_dense_mfma_kernel<N>;                                                                       \
    if (!allow_lds((const void*)kern, kDgSmem, lds_allowed)) return LOCMOE_ERR_HIP;                              \
    hipLaunchKernelGGL(kern, grid, dim3(kDgThreads), kDgSmem, s, (const uint16_t*)x, (const uint16_t*)Wg, g, T, \
                       d, E);                                                                                    \
  }
    if (nt == 1) LOCMOE_DG(1) else if (nt == 2) LOCMOE_DG(2) else if (nt == 3) LOCMOE_DG(3) else LOCMOE_DG(4)
#undef LOCMOE_DG
    return launch_status();
  }
  const dim3 grid(ceil_div(T, 4));
  if (desc->x_dtype == LOCMOE_BF16)
    hipLaunchKernelGGL(gate_dense_generic_kernel<true>, grid, dim3(256), 0, s, x, Wg, g, T, d, E);
  else
    hipLaunchKernelGGL(gate_dense_generic_kernel<false>, grid, dim3(256), 0, s, x, Wg, g, T, d, E);
  return launch_status();
}

extern "C" int locmoe_route_hash(const locmoe_desc* desc, const int32_t* key, uint32_t seed, int32_t* eid, float* w,
                                 int32_t* cnt, void* stream) {
  using namespace locmoe;
  if (!desc || !eid || !w || !cnt) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  hipStream_t s = as_stream(stream);
  const int T = desc->T, E = desc->E;
  hipLaunchKernelGGL(zero_i32_kernel, dim3(ceil_div(E, 256)), dim3(256), 0, s, cnt, E);
  int rc = launch_status();
  if (rc != LOCMOE_OK) return rc;
  hipLaunchKernelGGL(route_hash_kernel, dim3(ceil_div(T, kHashThreads * kHashPerThread)), dim3(kHashThreads),
                     (size_t)E * 4, s, key, seed * 0x9E3779B9u, eid, w, cnt, T, E);
  return launch_status();
}
