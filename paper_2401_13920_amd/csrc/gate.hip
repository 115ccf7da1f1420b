// GrAP gating value (Eq. 4): g[m,i] = mean of the i-th block of d/E consecutive features of
// token m.  Because blocks are contiguous and rows are contiguous, x is one flat array of
// 16-byte chunks and output number o (= m*E + i) is the mean of chunks [o*L, (o+1)*L) with
// L = (d/E)/VEC chunks per block: a flat segmented reduction, bandwidth-bound, no MFMA.
// With SQ the same pass also writes q[m,i] = sum of the squares of the block, from which the
// token's norm follows (the cosine between token and gating weight of Section 3.2.3 is
// g[m,i] * sqrt(d/E) / |x_m|).
#include "common.h"

namespace locmoe {
namespace {

constexpr int kGateThreads = 256;

template <bool BF16>
__device__ __forceinline__ float chunk_sum(const uint4& v) {
  return BF16 ? sum8_bf16(v) : sum4_f32(v);
}
template <bool BF16>
__device__ __forceinline__ float chunk_sumsq(const uint4& v) {
  return BF16 ? sumsq8_bf16(v) : sumsq4_f32(v);
}

// Power-of-two L <= 64: every lane loads U chunks (each load instruction of a wave is one
// contiguous 1 KiB), groups of L lanes are summed with DPP, the first lane of each group
// stores.  A block covers kGateThreads*U consecutive chunks.
template <bool BF16, int L, int U, bool SQ>
__global__ __launch_bounds__(kGateThreads) void gate_pow2_kernel(const uint4* __restrict__ x,
                                                                 float* __restrict__ g, float* __restrict__ qsq,
                                                                 long long chunks, float inv_blk) {
  const long long base = (long long)blockIdx.x * (kGateThreads * U) + threadIdx.x;
  uint4 v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const long long q = base + (long long)u * kGateThreads;
    v[u] = q < chunks ? nt_load16(x + q) : make_uint4(0, 0, 0, 0);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const long long q = base + (long long)u * kGateThreads;
    const float s = group_sum<L>(chunk_sum<BF16>(v[u]));
    if ((threadIdx.x & (L - 1)) == 0 && q < chunks) g[q / L] = s * inv_blk;
    if (SQ) {
      const float s2 = group_sum<L>(chunk_sumsq<BF16>(v[u]));
      if ((threadIdx.x & (L - 1)) == 0 && q < chunks) qsq[q / L] = s2;
    }
  }
}

// Any L <= kGateThreads*U: per-chunk sums go through LDS, then one thread per output adds its
// L partials in index order.  A block covers the largest multiple of L that fits.
template <bool BF16, int U, bool SQ>
__global__ __launch_bounds__(kGateThreads) void gate_lds_kernel(const uint4* __restrict__ x,
                                                                float* __restrict__ g, float* __restrict__ qsq,
                                                                long long outputs, int L, int out_per_block,
                                                                float inv_blk) {
  __shared__ float part[kGateThreads * U];
  __shared__ float part2[SQ ? kGateThreads * U : 1];
  const long long out0 = (long long)blockIdx.x * out_per_block;
  const int nout = (int)(outputs - out0 < out_per_block ? outputs - out0 : out_per_block);
  const int nchunk = nout * L;
  const uint4* src = x + out0 * L;
  uint4 v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int c = threadIdx.x + u * kGateThreads;
    v[u] = c < nchunk ? nt_load16(src + c) : make_uint4(0, 0, 0, 0);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    part[threadIdx.x + u * kGateThreads] = chunk_sum<BF16>(v[u]);
    if (SQ) part2[threadIdx.x + u * kGateThreads] = chunk_sumsq<BF16>(v[u]);
  }
  __syncthreads();
  for (int o = threadIdx.x; o < nout; o += kGateThreads) {
    float s = 0.f, s2 = 0.f;
    for (int j = 0; j < L; ++j) {
      s += part[o * L + j];
      if (SQ) s2 += part2[o * L + j];
    }
    g[out0 + o] = s * inv_blk;
    if (SQ) qsq[out0 + o] = s2;
  }
}

// Fallback for blocks that are not a whole number of 16-byte chunks, or longer than one LDS
// tile: one thread per output, scalar loads.
template <bool BF16, bool SQ>
__global__ __launch_bounds__(kGateThreads) void gate_scalar_kernel(const void* __restrict__ x,
                                                                   float* __restrict__ g, float* __restrict__ qsq,
                                                                   long long outputs, int blk, float inv_blk) {
  const long long o = (long long)blockIdx.x * kGateThreads + threadIdx.x;
  if (o >= outputs) return;
  float s = 0.f, s2 = 0.f;
  for (int j = 0; j < blk; ++j) {
    const float v = BF16 ? bf16_bits_to_f32(((const uint16_t*)x)[o * blk + j]) : ((const float*)x)[o * blk + j];
    s += v;
    if (SQ) s2 += v * v;
  }
  g[o] = s * inv_blk;
  if (SQ) qsq[o] = s2;
}

template <bool BF16, int L, bool SQ>
void launch_pow2(const void* x, float* g, float* q, long long chunks, float inv_blk, hipStream_t st) {
  constexpr int U = 8;
  const long long blocks = (chunks + kGateThreads * U - 1) / (kGateThreads * U);
  hipLaunchKernelGGL((gate_pow2_kernel<BF16, L, U, SQ>), dim3((unsigned)blocks), dim3(kGateThreads), 0, st,
                     (const uint4*)x, g, q, chunks, inv_blk);
}

template <bool BF16, bool SQ>
int gate_impl(const locmoe_desc* p, const void* x, float* g, float* q, hipStream_t st) {
  constexpr int VEC = BF16 ? 8 : 4;
  const int blk = p->d / p->E;
  const long long outputs = (long long)p->T * p->E;
  const float inv_blk = 1.0f / (float)blk;
  constexpr int U = 4;
  if (blk % VEC == 0 && blk / VEC <= kGateThreads * U) {
    const int L = blk / VEC;
    const long long chunks = outputs * L;
    switch (L) {
      case 1: launch_pow2<BF16, 1, SQ>(x, g, q, chunks, inv_blk, st); break;
      case 2: launch_pow2<BF16, 2, SQ>(x, g, q, chunks, inv_blk, st); break;
      case 4: launch_pow2<BF16, 4, SQ>(x, g, q, chunks, inv_blk, st); break;
      case 8: launch_pow2<BF16, 8, SQ>(x, g, q, chunks, inv_blk, st); break;
      case 16: launch_pow2<BF16, 16, SQ>(x, g, q, chunks, inv_blk, st); break;
      case 32: launch_pow2<BF16, 32, SQ>(x, g, q, chunks, inv_blk, st); break;
      case 64: launch_pow2<BF16, 64, SQ>(x, g, q, chunks, inv_blk, st); break;
      default: {
        const int opb = (kGateThreads * U) / L;
        const long long blocks = (outputs + opb - 1) / opb;
        hipLaunchKernelGGL((gate_lds_kernel<BF16, U, SQ>), dim3((unsigned)blocks), dim3(kGateThreads), 0, st,
                           (const uint4*)x, g, q, outputs, L, opb, inv_blk);
      }
    }
  } else {
    const long long blocks = (outputs + kGateThreads - 1) / kGateThreads;
    hipLaunchKernelGGL((gate_scalar_kernel<BF16, SQ>), dim3((unsigned)blocks), dim3(kGateThreads), 0, st, x, g,
                       q, outputs, blk, inv_blk);
  }
  return launch_status();
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_gate(const locmoe_desc* desc, const void* x, float* g, void* stream) {
  using namespace locmoe;
  if (!desc || !x || !g) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  return desc->x_dtype == LOCMOE_BF16 ? gate_impl<true, false>(desc, x, g, nullptr, as_stream(stream))
                                      : gate_impl<false, false>(desc, x, g, nullptr, as_stream(stream));
}

extern "C" int locmoe_gate_sq(const locmoe_desc* desc, const void* x, float* g, float* q, void* stream) {
  using namespace locmoe;
  if (!desc || !x || !g || !q) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  return desc->x_dtype == LOCMOE_BF16 ? gate_impl<true, true>(desc, x, g, q, as_stream(stream))
                                      : gate_impl<false, true>(desc, x, g, q, as_stream(stream));
}
