// Angles between tokens and gating weights: delta_{i,j} = cos(theta_{i,j}) of Section 3.2.3, and the
// measurement of Section 4.1 ("Analysis for Expert Capacity"): for the tokens routed to each expert, the
// histogram of their cosine to that expert's gating weight and to another expert's, and the smallest
// routed cosine, which is what the assumption in Section 3.2.3 calls delta.
// With the GrAP weight of Eq. 4 (|omega_i| = sqrt(E/d)), cos(x_m, omega_i) = g[m,i] * sqrt(d/E) / |x_m|;
// |x_m|^2 is the sum over i of the block sums of squares q[m,i] that locmoe_gate_sq writes.
// Integer atomics only (counts, and minima through an order-preserving integer image of the float):
// the results do not depend on the order in which tokens arrive.
#include <math.h>

#include "common.h"

namespace locmoe {
namespace {

constexpr int kAngThreads = 1024;        // 16 waves: each block gathers its tokens' counts in LDS first
constexpr int kAngTokens = 1024;         // tokens per block
constexpr int kAngLdsBytes = 48 * 1024;  // histograms larger than this are counted in global memory directly
constexpr float kNoCosine = 2.0f;        // what an expert without tokens reports: no cosine reaches it

// order-preserving map float -> int32 (and back), so that atomicMin on the image is a float minimum
__device__ __forceinline__ int ordered(float f) {
  const int i = __float_as_int(f);
  return i >= 0 ? i : i ^ 0x7FFFFFFF;
}
__device__ __forceinline__ float unordered(int i) { return __int_as_float(i >= 0 ? i : i ^ 0x7FFFFFFF); }

__global__ __launch_bounds__(256) void angle_init_kernel(int32_t* __restrict__ hist_self,
                                                         int32_t* __restrict__ hist_other,
                                                         int32_t* __restrict__ cmin_image, int cells, int E) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < cells) { hist_self[i] = 0; hist_other[i] = 0; }
  if (i < E) cmin_image[i] = ordered(kNoCosine);
}

__device__ __forceinline__ int bin_of(float c, int nbins) {
  const int b = (int)floorf((c + 1.0f) * 0.5f * (float)nbins);
  return min(nbins - 1, max(0, b));
}

// G lanes per token (a power of two <= 64) add the row of q in units of V floats: lane j takes units
// j, j+G, ...; the G partial sums are combined by a fixed butterfly.  With V = 4 and G = E/4 (E = 64:
// 16 lanes) one load instruction of a wave is 1 KiB of consecutive memory.  The first lane of the group
// then bins the token's two cosines.  Counts and minima are gathered per block in LDS and flushed with
// one atomic per non-empty cell (the per-expert minima sit in one cache line of global memory: sending
// every token's atomicMin there is what would bound the kernel otherwise).
template <int G, int V>
__global__ __launch_bounds__(kAngThreads) void angle_kernel(const float* __restrict__ g, const float* __restrict__ q,
                                                            const int32_t* __restrict__ eid,
                                                            float* __restrict__ c_self, float* __restrict__ c_other,
                                                            int32_t* __restrict__ hist_self,
                                                            int32_t* __restrict__ hist_other,
                                                            int32_t* __restrict__ cmin_image, int T, int E,
                                                            int shift, int nbins, float scale, int lds_cells) {
  extern __shared__ int32_t sm[];  // [E] images of the minima, then two histograms of lds_cells (or none)
  int32_t* s_min = sm;
  int32_t* s_self = sm + E;
  int32_t* s_other = s_self + lds_cells;
  for (int i = threadIdx.x; i < E; i += kAngThreads) s_min[i] = ordered(kNoCosine);
  for (int i = threadIdx.x; i < 2 * lds_cells; i += kAngThreads) s_self[i] = 0;
  __syncthreads();
  const int j = threadIdx.x % G, grp = threadIdx.x / G;
  const int units = E / V;
  const int m_end = min(T, (int)(blockIdx.x + 1) * kAngTokens);
#pragma unroll 2
  for (int m = blockIdx.x * kAngTokens + grp; m < m_end; m += kAngThreads / G) {
    const float* qr = q + (size_t)m * E;
    float part = 0.f;
    for (int u = j; u < units; u += G) {
      if (V == 4) {
        const float4 v = *(const float4*)(qr + 4 * u);
        part += (v.x + v.y) + (v.z + v.w);
      } else {
        part += qr[u];
      }
    }
    const float n2 = group_sum<G>(part);
    if (j == 0) {
      const int e = eid[m];
      int o = e + shift;
      o = o >= E ? o - E : o;
      const float inv = n2 > 0.f ? scale / sqrtf(n2) : 0.f;  // a zero token has no angle: cosines 0
      const float cs = g[(size_t)m * E + e] * inv, co = g[(size_t)m * E + o] * inv;
      if (c_self) c_self[m] = cs;
      if (c_other) c_other[m] = co;
      const int bs = e * nbins + bin_of(cs, nbins), bo = e * nbins + bin_of(co, nbins);
      if (lds_cells) {
        atomicAdd(&s_self[bs], 1);
        atomicAdd(&s_other[bo], 1);
      } else {
        atomicAdd(&hist_self[bs], 1);
        atomicAdd(&hist_other[bo], 1);
      }
      atomicMin(&s_min[e], ordered(cs));
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < lds_cells; i += kAngThreads) {
    const int a = s_self[i], b = s_other[i];
    if (a) atomicAdd(&hist_self[i], a);
    if (b) atomicAdd(&hist_other[i], b);
  }
  for (int i = threadIdx.x; i < E; i += kAngThreads) {
    const int v = s_min[i];
    // the global minimum only ever falls: a stale read can cost a needless atomic, never a lost one
    if (v < cmin_image[i]) atomicMin(&cmin_image[i], v);
  }
}

template <int V>
void launch_angles(int G, dim3 grid, size_t lds, hipStream_t s, const float* g, const float* q, const int32_t* eid,
                   float* c_self, float* c_other, int32_t* hist_self, int32_t* hist_other, int32_t* cmin_image, int T,
                   int E, int shift, int nbins, float scale, int lds_cells) {
#define LOCMOE_ANGLES(GG)                                                                                        \
  case GG:                                                                                                       \
    hipLaunchKernelGGL((angle_kernel<GG, V>), grid, dim3(kAngThreads), lds, s, g, q, eid, c_self, c_other,       \
                       hist_self, hist_other, cmin_image, T, E, shift, nbins, scale, lds_cells);                 \
    break;
  switch (G) {
    LOCMOE_ANGLES(1) LOCMOE_ANGLES(2) LOCMOE_ANGLES(4) LOCMOE_ANGLES(8) LOCMOE_ANGLES(16) LOCMOE_ANGLES(32)
    LOCMOE_ANGLES(64)
  }
#undef LOCMOE_ANGLES
}

// the minima back to floats, and delta_hat = the smallest of them
__global__ __launch_bounds__(1024) void angle_final_kernel(int32_t* __restrict__ cmin_image, float* __restrict__ stats,
                                                           int E) {
  __shared__ float red[1024];
  __shared__ int cnt[1024];
  float best = kNoCosine;
  int nonempty = 0;
  for (int i = threadIdx.x; i < E; i += 1024) {
    const float c = unordered(cmin_image[i]);
    ((float*)cmin_image)[i] = c;
    best = fminf(best, c);
    nonempty += c < kNoCosine ? 1 : 0;
  }
  red[threadIdx.x] = best;
  cnt[threadIdx.x] = nonempty;
  __syncthreads();
  for (int s = 512; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      red[threadIdx.x] = fminf(red[threadIdx.x], red[threadIdx.x + s]);
      cnt[threadIdx.x] += cnt[threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    stats[0] = red[0];           // delta_hat
    stats[1] = (float)cnt[0];    // experts that received tokens
    stats[2] = 0.f;
    stats[3] = 0.f;
  }
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_angle_stats(const locmoe_desc* desc, const float* g, const float* q, const int32_t* eid,
                                  int32_t shift, int32_t nbins, float* c_self, float* c_other, int32_t* hist_self,
                                  int32_t* hist_other, float* cmin, float* stats, void* stream) {
  using namespace locmoe;
  if (!desc || !g || !q || !eid || !hist_self || !hist_other || !cmin || !stats) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  if (nbins < 1 || nbins > 65536) return LOCMOE_ERR_ARG;
  const int E = desc->E;
  const int sh = ((shift % E) + E) % E;
  const int cells = E * nbins;
  hipStream_t s = as_stream(stream);
  hipLaunchKernelGGL(angle_init_kernel, dim3((unsigned)ceil_div(cells > E ? cells : E, 256)), dim3(256), 0, s,
                     hist_self, hist_other, (int32_t*)cmin, cells, E);
  const int V = E % 4 == 0 && (uintptr_t)q % 16 == 0 ? 4 : 1;
  int G = 1;
  while (G < 64 && 2 * G <= E / V) G *= 2;
  const int lds_cells = (size_t)(2 * cells + E) * 4 <= (size_t)kAngLdsBytes ? cells : 0;
  const size_t lds = (size_t)(2 * lds_cells + E) * 4;
  const dim3 grid((unsigned)ceil_div(desc->T, kAngTokens));
  const float scale = sqrtf((float)desc->d / (float)E);
  if (V == 4)
    launch_angles<4>(G, grid, lds, s, g, q, eid, c_self, c_other, hist_self, hist_other, (int32_t*)cmin, desc->T, E,
                     sh, nbins, scale, lds_cells);
  else
    launch_angles<1>(G, grid, lds, s, g, q, eid, c_self, c_other, hist_self, hist_other, (int32_t*)cmin, desc->T, E,
                     sh, nbins, scale, lds_cells);
  hipLaunchKernelGGL(angle_final_kernel, dim3(1), dim3(1024), 0, s, (int32_t*)cmin, stats, E);
  return launch_status();
}
