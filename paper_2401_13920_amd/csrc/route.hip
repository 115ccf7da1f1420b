// Top-1 routing (Eq. 2, Eq. 3) and the forward values of the auxiliary loss (Eq. 5) and the
// locality loss (Eq. 6).  One group of S lanes owns a token; reductions over the expert axis
// run on DPP / cross-lane permutes.  Every sum over tokens is formed from per-block partials in
// a fixed order (integer LDS atomics only, no floating-point atomics), so results are
// deterministic.
#include <math.h>

#include "common.h"

namespace locmoe {
namespace {

constexpr int kRouteThreads = 512;
constexpr int kTokPerGroup = 4;  // tokens a group loads before it starts reducing

// all-reduce (max value, lowest index) over aligned groups of S lanes
template <int S>
__device__ __forceinline__ void group_argmax(float& v, int& i) {
#define LOCMOE_STEP(OV, OI)                                \
  {                                                        \
    const float ov = (OV);                                 \
    const int oi = (OI);                                   \
    const bool take = ov > v || (ov == v && oi < i);       \
    v = take ? ov : v;                                     \
    i = take ? oi : i;                                     \
  }
  if (S >= 2) LOCMOE_STEP(dpp_f32<kDppXor1>(v), dpp_i32<kDppXor1>(i))
  if (S >= 4) LOCMOE_STEP(dpp_f32<kDppXor2>(v), dpp_i32<kDppXor2>(i))
  if (S >= 8) LOCMOE_STEP(dpp_f32<kDppHalfMirror>(v), dpp_i32<kDppHalfMirror>(i))
  if (S >= 16) LOCMOE_STEP(dpp_f32<kDppMirror>(v), dpp_i32<kDppMirror>(i))
  if (S >= 32) LOCMOE_STEP(__shfl_xor(v, 16), __shfl_xor(i, 16))
  if (S >= 64) LOCMOE_STEP(__shfl_xor(v, 32), __shfl_xor(i, 32))
#undef LOCMOE_STEP
}

struct RouteWs {
  int32_t* cnt;    // [blocks][E]
  float* psum;     // [blocks][E]
  int32_t* home;   // [blocks][N]
  int32_t* local;  // [blocks]
};

__host__ __device__ inline RouteWs route_ws(void* ws, int E, int N) {
  RouteWs r;
  char* p = (char*)ws;
  r.cnt = (int32_t*)p;   p += (size_t)kRouteMaxBlocks * E * 4;
  r.psum = (float*)p;    p += (size_t)kRouteMaxBlocks * E * 4;
  r.home = (int32_t*)p;  p += (size_t)kRouteMaxBlocks * N * 4;
  r.local = (int32_t*)p;
  return r;
}

template <int S, int EPL>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(
    const float* __restrict__ g, const float* __restrict__ eps, const int32_t* __restrict__ home,
    const int32_t* __restrict__ e2n, int32_t* __restrict__ eid, float* __restrict__ w, void* ws, int T,
    int E, int N, int relu, int tokens_per_block) {
  constexpr int G = kRouteThreads / S;  // groups (tokens in flight) per block
  extern __shared__ char smem[];
  int32_t* hist = (int32_t*)smem;            // [E]
  int32_t* hhist = hist + E;                 // [N]
  int32_t* local = hhist + N;                // [1]
  float* pacc = (float*)(local + 1);         // [G][E]
  for (int i = threadIdx.x; i < E + N + 1; i += kRouteThreads) hist[i] = 0;
  __syncthreads();

  const int grp = threadIdx.x / S, j = threadIdx.x % S;
  const int per_node = E / N;  // used only when e2n is NULL (then E % N == 0)
  float epsv[EPL];
#pragma unroll
  for (int k = 0; k < EPL; ++k) {
    const int i = j + k * S;
    epsv[k] = (eps && i < E) ? eps[i] : 0.f;
  }
  float acc[EPL];
#pragma unroll
  for (int k = 0; k < EPL; ++k) acc[k] = 0.f;

  const int tok0 = blockIdx.x * tokens_per_block;
  const int tok1 = min(T, tok0 + tokens_per_block);
  // the loads of the next batch of tokens are issued before the current batch is reduced
  // (the tokens' home nodes come with the batch: fetched where they are used, behind the arg-max, each was a
  // memory round trip of its own on the critical path)
  float v[kTokPerGroup][EPL], nxt[kTokPerGroup][EPL];
  int hv[kTokPerGroup], hnxt[kTokPerGroup];
  auto load_batch = [&](float (&dst)[kTokPerGroup][EPL], int (&hdst)[kTokPerGroup], int base) {
#pragma unroll
    for (int t = 0; t < kTokPerGroup; ++t) {
      const int m = base + t * G + grp;
#pragma unroll
      for (int k = 0; k < EPL; ++k) {
        const int i = j + k * S;
        dst[t][k] = (m < tok1 && i < E) ? g[(size_t)m * E + i] : -INFINITY;
      }
      hdst[t] = (home && j == 0 && m < tok1) ? home[m] : 0;
    }
  };
  load_batch(nxt, hnxt, tok0);
  for (int base = tok0; base < tok1; base += G * kTokPerGroup) {
#pragma unroll
    for (int t = 0; t < kTokPerGroup; ++t) {
#pragma unroll
      for (int k = 0; k < EPL; ++k) v[t][k] = nxt[t][k];
      hv[t] = hnxt[t];
    }
    load_batch(nxt, hnxt, base + G * kTokPerGroup);
#pragma unroll
    for (int t = 0; t < kTokPerGroup; ++t) {
      const int m = base + t * G + grp;
      float best = -INFINITY;
      int bi = 0x7FFFFFFF;
#pragma unroll
      for (int k = 0; k < EPL; ++k) {
        const int i = j + k * S;
        float x = v[t][k] + epsv[k];           // G = g + eps, float32
        if (relu) x = fmaxf(x, 0.f);           // ReLU as printed below Eq. 3
        x = i < E ? x : -INFINITY;
        v[t][k] = x;
        if (x > best) { best = x; bi = i; }    // strict: lowest index wins ties
      }
      group_argmax<S>(best, bi);
      float z[EPL], zs = 0.f;
#pragma unroll
      for (int k = 0; k < EPL; ++k) {
        z[k] = (j + k * S) < E ? expf(v[t][k] - best) : 0.f;
        zs += z[k];
      }
      zs = group_sum<S>(zs);
      const float inv = 1.0f / zs;
      if (m < tok1) {
#pragma unroll
        for (int k = 0; k < EPL; ++k) acc[k] += z[k] * inv;
        if (j == 0) {
          eid[m] = bi;
          w[m] = inv;  // exp(0) / sum
          atomicAdd(&hist[bi], 1);
          if (home) {
            const int hn = hv[t];
            atomicAdd(&hhist[hn], 1);
            const int node = e2n ? e2n[bi] : bi / per_node;
            if (node == hn) atomicAdd(local, 1);
          }
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < EPL; ++k) {
    const int i = j + k * S;
    if (i < E) pacc[grp * E + i] = acc[k];
  }
  __syncthreads();
  RouteWs r = route_ws(ws, E, N);
  for (int i = threadIdx.x; i < E; i += kRouteThreads) {
    float s = 0.f;
    for (int q = 0; q < G; ++q) s += pacc[q * E + i];
    r.psum[(size_t)blockIdx.x * E + i] = s;
    r.cnt[(size_t)blockIdx.x * E + i] = hist[i];
  }
  for (int i = threadIdx.x; i < N; i += kRouteThreads) r.home[(size_t)blockIdx.x * N + i] = hhist[i];
  if (threadIdx.x == 0) r.local[blockIdx.x] = *local;
}

constexpr int kFinThreads = 1024;
constexpr int kFinWaves = kFinThreads / kWave;

// Sums (and one maximum) over the block of NQ doubles per thread, in a fixed order: a butterfly inside each wave
// (lane i adds lane i ^ o for o = 32 .. 1), the sixteen wave results through LDS, added in wave order by every
// thread.  Two barriers for all NQ quantities together.
template <int NQ>
__device__ __forceinline__ void block_sums(double (&v)[NQ], double& vmax, double (*part)[kFinWaves]) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) v[q] += __shfl_xor(v[q], o);
    vmax = fmax(vmax, __shfl_xor(vmax, o));
  }
  const int wave = threadIdx.x / kWave;
  if (threadIdx.x % kWave == 0) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) part[q][wave] = v[q];
    part[NQ][wave] = vmax;
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kFinWaves; ++w) t += part[q][w];
    v[q] = t;
  }
  double m = part[NQ][0];
#pragma unroll
  for (int w = 1; w < kFinWaves; ++w) m = fmax(m, part[NQ][w]);
  vmax = m;
}

// One block: column sums of the per-block partials, then the scalars of Eq. 5 / Eq. 6.
__global__ __launch_bounds__(kFinThreads) void route_finalize_kernel(
    void* ws, const int32_t* __restrict__ e2n, int has_home, int32_t* __restrict__ cnt,
    float* __restrict__ Psum, float* __restrict__ stats, int nb, int T, int E, int N, float alpha, float mu) {
  __shared__ double part[6][kFinWaves];
  __shared__ double dpart[kFinThreads];
  __shared__ int32_t ipart[kFinThreads];
  __shared__ int32_t s_cnt[1024];
  __shared__ double s_P[1024];
  __shared__ int32_t s_home[1024];
  __shared__ int32_t s_pernode[1024];
  RouteWs r = route_ws(ws, E, N);
  const int tid = threadIdx.x;
  if (tid < N) { s_home[tid] = 0; s_pernode[tid] = 0; }
  int local = 0;
  int32_t hi = 0;
  {  // cnt and Psum: thread (rb, e) adds rows rb, rb+R, ... in order; then the row groups are added in order.
     // The home-node counts the same way.
    const int R = kFinThreads / E;
    const int e = tid % E, rb = tid / E;
    int32_t ci = 0;
    double ps = 0.0;
    // Loads are unconditional (rows past the end re-read the thread's first row and are not added) and all of
    // a round's loads - counts, probability sums, home counts, locality counts - are issued before the first
    // is used: the partials were written by other XCDs, every dependent round trip costs microseconds, and with
    // the bound inside the loop every load waited for the one before it.
    constexpr int U = 32, UH = 8;
    const int Rn = kFinThreads / N;
    const int nu = tid % N, rn = tid / N;
    const bool cols = rb < R && rb < nb, hcols = has_home && rn < Rn && rn < nb;
    for (int b0 = 0; b0 < nb; b0 += U * R) {
      int32_t cv[U];
      float pv[U];
      int32_t hvv[UH];
      if (cols) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int b = b0 + rb + u * R;
          const size_t at = (size_t)(b < nb ? b : rb) * E + e;
          cv[u] = r.cnt[at];
          pv[u] = r.psum[at];
        }
      }
      const bool hround = hcols && b0 == 0;   // the home counts go with the first round (looped below if they are many)
      if (hround) {
#pragma unroll
        for (int u = 0; u < UH; ++u) {
          const int b = rn + u * Rn;
          hvv[u] = r.home[(size_t)(b < nb ? b : rn) * N + nu];
        }
      }
      if (has_home && b0 == 0)
        for (int b = tid; b < nb; b += kFinThreads) local += r.local[b];
      if (cols) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const bool live = b0 + rb + u * R < nb;
          ci += live ? cv[u] : 0;
          ps += live ? (double)pv[u] : 0.0;
        }
      }
      if (hround) {
#pragma unroll
        for (int u = 0; u < UH; ++u) hi += (rn + u * Rn < nb) ? hvv[u] : 0;
      }
    }
    if (hcols)  // home counts beyond the first UH rows of this thread (few nodes per thread group: rare)
      for (int b = rn + UH * Rn; b < nb; b += Rn) hi += r.home[(size_t)b * N + nu];
    ipart[tid] = ci;
    dpart[tid] = ps;
    __syncthreads();
    if (tid < E) {
      int32_t c = 0;
      double p = 0.0;
      for (int q = 0; q < R; ++q) { c += ipart[q * E + tid]; p += dpart[q * E + tid]; }
      s_cnt[tid] = c;
      s_P[tid] = p;
      cnt[tid] = c;
      Psum[tid] = (float)p;
    }
    if (has_home) {  // integer adds: any order gives the same counts
      if (hi) atomicAdd(&s_home[tid % N], hi);
      if (tid < E) atomicAdd(&s_pernode[e2n ? e2n[tid] : tid / (E / N)], 1);
    }
    __syncthreads();
  }
  // Eq. 5: L_aux = alpha * n * sum_i f_i P_i
  double q[5] = {0.0, 0.0, 0.0, (double)local, 0.0};  // f P, KL(f || D_l), KL(P || D_l) terms, local tokens, empty experts
  double mx = 0.0;
  if (tid < E) {
    const double f = (double)s_cnt[tid] / T, P = s_P[tid] / T;
    q[0] = f * P;
    mx = (double)s_cnt[tid];
    q[4] = s_cnt[tid] == 0 ? 1.0 : 0.0;
    if (has_home) {
      // Eq. 6 over experts: D_l[i] = T_node(i) / (T * experts on node(i))
      const int nu = e2n ? e2n[tid] : tid / (E / N);
      const double Dl = (double)s_home[nu] / ((double)T * (double)s_pernode[nu]);
      if (f > 0.0) q[1] = Dl > 0.0 ? f * log(f / Dl) : INFINITY;
      if (P > 0.0) q[2] = Dl > 0.0 ? P * log(P / Dl) : INFINITY;
    }
  }
  block_sums<5>(q, mx, part);
  if (tid == 0) {
    stats[0] = (float)((double)alpha * E * q[0]);
    stats[1] = (float)q[1];
    stats[2] = (float)q[2];
    stats[3] = (float)((double)mu * q[1]);
    stats[4] = (float)(q[3] / T);
    stats[5] = (float)mx;
    stats[6] = (float)q[4];
    stats[7] = 0.f;
  }
}

template <int S, int EPL>
void launch_route(const locmoe_desc* p, const float* g, const float* eps, const int32_t* home,
                  const int32_t* e2n, int32_t* eid, float* w, void* ws, int nb, int tpb, hipStream_t st) {
  constexpr int G = kRouteThreads / S;
  const size_t smem = (size_t)(p->E + p->N + 1) * 4 + (size_t)G * p->E * 4;
  hipLaunchKernelGGL((route_kernel<S, EPL>), dim3(nb), dim3(kRouteThreads), smem, st, g, eps, home, e2n, eid,
                     w, ws, p->T, p->E, p->N, p->relu, tpb);
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_route(const locmoe_desc* desc, const float* g, const float* eps, const int32_t* home,
                            const int32_t* e2n, int32_t* eid, float* w, int32_t* cnt, float* Psum,
                            float* stats, void* ws, size_t ws_bytes, void* stream) {
  using namespace locmoe;
  if (!desc || !g || !eid || !w || !cnt || !Psum || !stats) return LOCMOE_ERR_NULL;
  int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  if (!e2n && desc->E % desc->N != 0) return LOCMOE_ERR_SHAPE;
  if (!ws || ws_bytes < locmoe_workspace_bytes(desc)) return LOCMOE_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  const int E = desc->E;
  // lanes per token: the whole expert axis up to 16 experts; beyond that, up to 128 experts, 16 lanes with
  // several experts each (four tokens per wave side by side: the cross-lane reductions, which dominate the
  // instruction count, shrink from six steps to four and are shared by four tokens); one wave per token above
  int S = 4;
  while (S < E && S < 16) S *= 2;
  if (E > 128) S = 64;
  const int G = kRouteThreads / S;
  const int step = G * kTokPerGroup;
  int tpb = ceil_div(desc->T, kRouteMaxBlocks);
  tpb = ceil_div(tpb, step) * step;
  const int nb = ceil_div(desc->T, tpb);
  const int epl = ceil_div(E, S);
#define LOCMOE_ROUTE(SS, EE) launch_route<SS, EE>(desc, g, eps, home, e2n, eid, w, ws, nb, tpb, s)
  if (S == 4) LOCMOE_ROUTE(4, 1);
  else if (S == 8) LOCMOE_ROUTE(8, 1);
  else if (S == 16 && epl == 1) LOCMOE_ROUTE(16, 1);
  else if (S == 16 && epl == 2) LOCMOE_ROUTE(16, 2);
  else if (S == 16 && epl <= 4) LOCMOE_ROUTE(16, 4);
  else if (S == 16) LOCMOE_ROUTE(16, 8);
  else if (epl <= 4) LOCMOE_ROUTE(64, 4);
  else if (epl <= 8) LOCMOE_ROUTE(64, 8);
  else LOCMOE_ROUTE(64, 16);
#undef LOCMOE_ROUTE
  st = launch_status();
  if (st != LOCMOE_OK) return st;
  hipLaunchKernelGGL(route_finalize_kernel, dim3(1), dim3(kFinThreads), 0, s, ws, e2n, home ? 1 : 0, cnt, Psum,
                     stats, nb, desc->T, E, desc->N, desc->alpha, desc->mu);
  return launch_status();
}
