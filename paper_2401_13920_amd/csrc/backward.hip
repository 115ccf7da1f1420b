// Backward of the bandwidth-bound steps of the layer: the chain rule through Eq. 1 (combine under top-1),
// Eq. 3 with the ReLU printed below it, Eq. 4 (GrAP) and the two batch losses of Section 3.2.2
// (Eq. 5 with f held fixed; Eq. 6 differentiated through the mean router probability P).
//   locmoe_combine_bwd   dout[slot_m] = w_m dy_m,  dw_m = <dy_m, out[slot_m]>
//   locmoe_route_bwd     dp = [i = e*] dw + coef,  dG = p (dp - <p, dp>),  dg = dG where g + eps > 0
//   locmoe_dispatch_bwd  dx_m = dsend[slot_m] (kept) + (E/d) dg[m, block(j)]
// Every output element is written exactly once by one lane, sums run in a fixed order: no atomics in the
// results, bitwise repeatable.
#include <math.h>

#include <algorithm>

#include "common.h"

namespace locmoe {
namespace {

constexpr int kBwdThreads = 256;

template <bool BF16>
__device__ __forceinline__ float dot16(const uint4& a, const uint4& b) {
  if (BF16) {
    const uint32_t* p = &a.x;
    const uint32_t* q = &b.x;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s = fmaf(bf16_bits_to_f32(p[i] & 0xFFFFu), bf16_bits_to_f32(q[i] & 0xFFFFu), s);
      s = fmaf(__uint_as_float(p[i] & 0xFFFF0000u), __uint_as_float(q[i] & 0xFFFF0000u), s);
    }
    return s;
  }
  float s = __uint_as_float(a.x) * __uint_as_float(b.x);
  s = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), s);
  s = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), s);
  return fmaf(__uint_as_float(a.w), __uint_as_float(b.w), s);
}

// One wave per token row.  A dropped token reads nothing and gets dw = 0.
template <bool BF16>
__global__ __launch_bounds__(kBwdThreads) void combine_bwd_kernel(const uint4* __restrict__ dy,
                                                                  const uint4* __restrict__ out,
                                                                  const int32_t* __restrict__ slot,
                                                                  const float* __restrict__ w,
                                                                  uint4* __restrict__ dout, float* __restrict__ dw,
                                                                  int T, int chunks) {
  const int m = blockIdx.x * (kBwdThreads / kWave) + threadIdx.x / kWave;
  if (m >= T) return;
  const int l = threadIdx.x % kWave;
  const int s = slot[m];
  if (s < 0) {
    if (l == 0) dw[m] = 0.f;
    return;
  }
  const float wm = w[m];
  const uint4* a = dy + (size_t)m * chunks;
  const uint4* b = out + (size_t)s * chunks;
  uint4* dst = dout + (size_t)s * chunks;
  float acc = 0.f;
  constexpr int U = 4;
  int c = l;
  for (; c + (U - 1) * kWave < chunks; c += U * kWave) {
    uint4 va[U], vb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) { va[u] = nt_load16(a + c + u * kWave); vb[u] = nt_load16(b + c + u * kWave); }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc += dot16<BF16>(va[u], vb[u]);
      nt_store16(scale16<BF16>(va[u], wm), dst + c + u * kWave);
    }
  }
  for (; c < chunks; c += kWave) {
    const uint4 va = nt_load16(a + c), vb = nt_load16(b + c);
    acc += dot16<BF16>(va, vb);
    nt_store16(scale16<BF16>(va, wm), dst + c);
  }
  acc = group_sum<kWave>(acc);
  if (l == 0) dw[m] = acc;
}

// Tokens per home node, first pass: every block counts its share of the tokens in LDS (integer atomics: the
// order does not matter) and writes one row of a [blocks, N] matrix.  The matrix lives in the front of dg, which
// locmoe_route_bwd writes only afterwards (no entry point of the backward takes a workspace).
constexpr int kHomeThreads = 256;
__global__ __launch_bounds__(kHomeThreads) void route_bwd_home_kernel(const int32_t* __restrict__ home,
                                                                      int32_t* __restrict__ part, int T, int N,
                                                                      int per_block) {
  extern __shared__ int32_t hist[];
  for (int i = threadIdx.x; i < N; i += kHomeThreads) hist[i] = 0;
  __syncthreads();
  const int m0 = blockIdx.x * per_block, m1 = min(T, m0 + per_block);
  for (int m = m0 + threadIdx.x; m < m1; m += kHomeThreads) atomicAdd(&hist[home[m]], 1);
  __syncthreads();
  for (int i = threadIdx.x; i < N; i += kHomeThreads) part[(size_t)blockIdx.x * N + i] = hist[i];
}

// One block: column sums of that matrix, experts per node, then the per-expert coefficient that every token's
// dp receives: alpha n f_i / T (Eq. 5, f fixed) + mu (ln(P_i / D_l[i]) + 1) / T (Eq. 6 through P).
__global__ __launch_bounds__(1024) void route_bwd_coef_kernel(const int32_t* __restrict__ part, int nblk,
                                                              const int32_t* __restrict__ e2n,
                                                              const int32_t* __restrict__ cnt,
                                                              const float* __restrict__ Psum,
                                                              float* __restrict__ coef, int T, int E, int N,
                                                              float alpha, float mu) {
  __shared__ int32_t s_home[1024];
  __shared__ int32_t s_pernode[1024];
  const int tid = threadIdx.x;
  if (tid < N) { s_home[tid] = 0; s_pernode[tid] = 0; }
  __syncthreads();
  if (part) {
    // thread (rg, nu) adds rows rg, rg + R, ... of column nu: eight unconditional loads at a time (rows past the
    // end re-read row rg and are not added), so that a batch is in flight together
    const int R = 1024 / N, nu = tid % N, rg = tid / N;
    if (rg < R && rg < nblk) {
      int32_t sum = 0;
      for (int q0 = rg; q0 < nblk; q0 += 8 * R) {
        int32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int q = q0 + u * R;
          v[u] = part[(size_t)(q < nblk ? q : rg) * N + nu];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += (q0 + u * R < nblk) ? v[u] : 0;
      }
      if (sum) atomicAdd(&s_home[nu], sum);
    }
    if (tid < E) atomicAdd(&s_pernode[e2n ? e2n[tid] : tid / (E / N)], 1);
  }
  __syncthreads();
  if (tid < E) {
    double c = (double)alpha * E * ((double)cnt[tid] / T) / T;
    if (part && mu != 0.f) {
      const int nu = e2n ? e2n[tid] : tid / (E / N);
      const double Dl = (double)s_home[nu] / ((double)T * (double)s_pernode[nu]);
      const double P = (double)Psum[tid] / T;
      c += (double)mu * (log(P / Dl) + 1.0) / T;
    }
    coef[tid] = (float)c;
  }
}

// G lanes per token; lane j owns experts j, j+G, ...  The softmax is recomputed from g as the forward did.
template <int G>
__global__ __launch_bounds__(kBwdThreads) void route_bwd_kernel(const float* __restrict__ g,
                                                                const float* __restrict__ eps,
                                                                const int32_t* __restrict__ eid,
                                                                const float* __restrict__ dw,
                                                                const float* __restrict__ coef,
                                                                float* __restrict__ dg, int T, int E, int relu) {
  const int m = blockIdx.x * (kBwdThreads / G) + threadIdx.x / G;
  if (m >= T) return;  // whole groups leave together
  const int j = threadIdx.x % G;
  const float* gr = g + (size_t)m * E;
  float best = -INFINITY;
  for (int i = j; i < E; i += G) {
    float s = gr[i] + (eps ? eps[i] : 0.f);
    if (relu) s = fmaxf(s, 0.f);
    best = fmaxf(best, s);
  }
#pragma unroll
  for (int o = G / 2; o > 0; o >>= 1) best = fmaxf(best, __shfl_xor(best, o));
  const int e = eid[m];
  const float dwm = dw[m];
  float zs = 0.f, zc = 0.f;  // sum of exp, sum of exp * dp
  for (int i = j; i < E; i += G) {
    float s = gr[i] + (eps ? eps[i] : 0.f);
    if (relu) s = fmaxf(s, 0.f);
    const float z = expf(s - best);
    zs += z;
    zc = fmaf(z, coef[i] + (i == e ? dwm : 0.f), zc);
  }
  zs = group_sum<G>(zs);
  zc = group_sum<G>(zc);
  const float inv = 1.0f / zs;
  const float inner = zc * inv;  // <p, dp>
  for (int i = j; i < E; i += G) {
    const float raw = gr[i] + (eps ? eps[i] : 0.f);
    const float s = relu ? fmaxf(raw, 0.f) : raw;
    const float p = expf(s - best) * inv;
    const float v = p * (coef[i] + (i == e ? dwm : 0.f) - inner);
    dg[(size_t)m * E + i] = (relu && !(raw > 0.f)) ? 0.f : v;  // ReLU'(0) = 0
  }
}

// One wave per token row: the gradient row that comes back from the expert plus the GrAP term.
// VEC_BLOCK: a 16-byte chunk lies inside one GrAP block (block length a multiple of the chunk's elements).
template <bool BF16, bool VEC_BLOCK>
__global__ __launch_bounds__(kBwdThreads) void dispatch_bwd_kernel(const uint4* __restrict__ dsend,
                                                                   const int32_t* __restrict__ slot,
                                                                   const float* __restrict__ dg,
                                                                   uint4* __restrict__ dx, int T, int chunks,
                                                                   int E, int blk, float scale) {
  constexpr int VEC = BF16 ? 8 : 4;
  const int m = blockIdx.x * (kBwdThreads / kWave) + threadIdx.x / kWave;
  if (m >= T) return;
  const int l = threadIdx.x % kWave;
  const int s = slot[m];
  const uint4* src = s >= 0 ? dsend + (size_t)s * chunks : nullptr;
  const float* dgr = dg + (size_t)m * E;
  uint4* dst = dx + (size_t)m * chunks;
  for (int c = l; c < chunks; c += kWave) {
    const uint4 v = src ? nt_load16(src + c) : make_uint4(0, 0, 0, 0);
    float a[VEC];
    if (BF16) {
      const uint32_t* p = &v.x;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[2 * i] = bf16_bits_to_f32(p[i] & 0xFFFFu);
        a[2 * i + 1] = __uint_as_float(p[i] & 0xFFFF0000u);
      }
    } else {
      a[0] = __uint_as_float(v.x); a[1] = __uint_as_float(v.y);
      a[2] = __uint_as_float(v.z); a[3] = __uint_as_float(v.w);
    }
    if (VEC_BLOCK) {
      const float t = scale * dgr[(c * VEC) / blk];
#pragma unroll
      for (int i = 0; i < VEC; ++i) a[i] += t;
    } else {
#pragma unroll
      for (int i = 0; i < VEC; ++i) a[i] = fmaf(scale, dgr[(c * VEC + i) / blk], a[i]);
    }
    uint4 r;
    if (BF16) {
      r = make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]),
                     pack_bf16x2(a[6], a[7]));
    } else {
      r = make_uint4(__float_as_uint(a[0]), __float_as_uint(a[1]), __float_as_uint(a[2]), __float_as_uint(a[3]));
    }
    nt_store16(r, dst + c);
  }
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_combine_bwd(const locmoe_desc* desc, const void* dy, const void* out, const int32_t* slot,
                                  const float* w, void* dout, float* dw, void* stream) {
  using namespace locmoe;
  if (!desc || !dy || !out || !slot || !w || !dout || !dw) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  const bool bf = desc->x_dtype == LOCMOE_BF16;
  const int chunks = desc->d * (bf ? 2 : 4) / 16;
  const dim3 grid((unsigned)ceil_div(desc->T, kBwdThreads / kWave));
  if (bf)
    hipLaunchKernelGGL(combine_bwd_kernel<true>, grid, dim3(kBwdThreads), 0, as_stream(stream), (const uint4*)dy,
                       (const uint4*)out, slot, w, (uint4*)dout, dw, desc->T, chunks);
  else
    hipLaunchKernelGGL(combine_bwd_kernel<false>, grid, dim3(kBwdThreads), 0, as_stream(stream), (const uint4*)dy,
                       (const uint4*)out, slot, w, (uint4*)dout, dw, desc->T, chunks);
  return launch_status();
}

extern "C" int locmoe_route_bwd(const locmoe_desc* desc, const float* g, const float* eps, const int32_t* home,
                                const int32_t* e2n, const int32_t* eid, const int32_t* cnt, const float* Psum,
                                const float* dw, float* coef, float* dg, void* stream) {
  using namespace locmoe;
  if (!desc || !g || !eid || !cnt || !Psum || !dw || !coef || !dg) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  if (!e2n && desc->E % desc->N != 0) return LOCMOE_ERR_SHAPE;
  hipStream_t s = as_stream(stream);
  const int E = desc->E, T = desc->T;
  // tokens per home node: partial counts of up to 256 blocks in the front of dg (T E words; N <= E, so a matrix
  // of at most T rows always fits), summed by the coefficient kernel before dg itself is written
  const int N = desc->N;
  int32_t* part = nullptr;
  int nblk = 0;
  if (home) {
    const long long fit = (long long)T * E / N;
    nblk = (int)std::min<long long>(std::min<long long>(256, ceil_div(T, kHomeThreads)), fit);
    const int per_block = ceil_div(T, nblk);
    nblk = ceil_div(T, per_block);
    part = (int32_t*)dg;
    hipLaunchKernelGGL(route_bwd_home_kernel, dim3(nblk), dim3(kHomeThreads), (size_t)N * 4, s, home, part, T, N,
                       per_block);
  }
  hipLaunchKernelGGL(route_bwd_coef_kernel, dim3(1), dim3(1024), 0, s, part, nblk, e2n, cnt, Psum, coef, T, E, N,
                     desc->alpha, desc->mu);
  int G = 1;
  while (G < 64 && 2 * G <= E) G *= 2;
#define LOCMOE_ROUTE_BWD(GG)                                                                                      \
  case GG:                                                                                                        \
    hipLaunchKernelGGL(route_bwd_kernel<GG>, dim3((unsigned)ceil_div(T, kBwdThreads / GG)), dim3(kBwdThreads), 0, \
                       s, g, eps, eid, dw, coef, dg, T, E, desc->relu);                                           \
    break;
  switch (G) {
    LOCMOE_ROUTE_BWD(1) LOCMOE_ROUTE_BWD(2) LOCMOE_ROUTE_BWD(4) LOCMOE_ROUTE_BWD(8) LOCMOE_ROUTE_BWD(16)
    LOCMOE_ROUTE_BWD(32) LOCMOE_ROUTE_BWD(64)
  }
#undef LOCMOE_ROUTE_BWD
  return launch_status();
}

extern "C" int locmoe_dispatch_bwd(const locmoe_desc* desc, const void* dsend, const int32_t* slot, const float* dg,
                                   void* dx, void* stream) {
  using namespace locmoe;
  if (!desc || !dsend || !slot || !dg || !dx) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  const bool bf = desc->x_dtype == LOCMOE_BF16;
  const int vec = bf ? 8 : 4;
  const int chunks = desc->d / vec;
  const int blk = desc->d / desc->E;
  const float scale = (float)desc->E / (float)desc->d;
  const dim3 grid((unsigned)ceil_div(desc->T, kBwdThreads / kWave));
  hipStream_t s = as_stream(stream);
#define LOCMOE_DISPATCH_BWD(BF, VB)                                                                          \
  hipLaunchKernelGGL((dispatch_bwd_kernel<BF, VB>), grid, dim3(kBwdThreads), 0, s, (const uint4*)dsend, slot, dg, \
                     (uint4*)dx, desc->T, chunks, desc->E, blk, scale)
  if (bf) {
    if (blk % vec == 0) LOCMOE_DISPATCH_BWD(true, true);
    else LOCMOE_DISPATCH_BWD(true, false);
  } else {
    if (blk % vec == 0) LOCMOE_DISPATCH_BWD(false, true);
    else LOCMOE_DISPATCH_BWD(false, false);
  }
#undef LOCMOE_DISPATCH_BWD
  return launch_status();
}
