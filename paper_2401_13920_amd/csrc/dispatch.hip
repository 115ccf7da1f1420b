// Capacity-bounded stable dispatch (capacity: Section 3.2.3).
//   1. dispatch_hist_kernel   per block of 1024 tokens: count of tokens per expert
//   2. dispatch_slots_kernel  every block re-derives, from the [blocks,E] count matrix, the
//      tokens before it per expert and the totals, hence kept[], the buffer order and the
//      segment offsets; then ranks its own tokens (wave ballots + ordered wave prefixes)
//   3. dispatch_copy_kernel   send[r,:] = x[row_token[r],:] for r < K, 16-byte vectors
// Integer-only; LDS integer atomics appear only where the result does not depend on their
// order, so slots are bit-identical from run to run.
#include <atomic>

#include "common.h"

namespace locmoe {
namespace {

// Scratch of locmoe_dispatch_static: the [blocks, E] count matrix lives in this array instead of a caller
// workspace.  Host code never uses the array's name as an address: static_scratch() asks the runtime for the
// device address once per device and hands that pointer to the kernels.
constexpr size_t kStaticScratchBytes = size_t(1) << 20;  // 262 144 counts: blocks of 1024 tokens x experts
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (each device holds its own copy), nullptr if the runtime
// refuses.  Asked once per device; later calls read the cached pointer.
void* static_scratch() {
  static std::atomic<void*> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  void* ptr = cached[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    cached[dev].store(ptr, std::memory_order_release);
  }
  return ptr;
}

constexpr int kDispThreads = 256;
constexpr int kDispWaves = kDispThreads / kWave;
constexpr int kTokPerWave = kDispatchTokensPerBlock / kDispWaves;  // contiguous tokens per wave
constexpr int kIter = kTokPerWave / kWave;

// Orders this wave's LDS accesses before the call against those after it, for all lanes.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(kDispThreads) void dispatch_hist_kernel(const int32_t* __restrict__ eid,
                                                                     int32_t* __restrict__ blockcnt, int T,
                                                                     int E) {
  extern __shared__ int32_t hist[];
  for (int i = threadIdx.x; i < E; i += kDispThreads) hist[i] = 0;
  __syncthreads();
  const int base = blockIdx.x * kDispatchTokensPerBlock;
#pragma unroll
  for (int k = 0; k < kDispatchTokensPerBlock / kDispThreads; ++k) {
    const int m = base + k * kDispThreads + threadIdx.x;
    if (m < T) atomicAdd(&hist[eid[m]], 1);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < E; i += kDispThreads) blockcnt[(size_t)blockIdx.x * E + i] = hist[i];
}

// LDS layout of the slots kernel (ints): off[E] tot[E] node[E] rank[E] seg[E+1] wcnt[waves][E]
__global__ __launch_bounds__(kDispThreads) void dispatch_slots_kernel(
    const int32_t* __restrict__ eid, const int32_t* __restrict__ e2n, const int32_t* __restrict__ blockcnt,
    int32_t* __restrict__ pos, int32_t* __restrict__ slot, int32_t* __restrict__ kept,
    int32_t* __restrict__ seg_off, int32_t* __restrict__ node_off, int32_t* __restrict__ buf_expert,
    int32_t* __restrict__ row_token, int T, int E, int N, int C, int nblocks, int nbits) {
  extern __shared__ int32_t sm[];
  int32_t* off = sm;
  int32_t* tot = off + E;
  int32_t* node = tot + E;
  int32_t* rank = node + E;
  int32_t* seg = rank + E;  // [E+1], indexed by buffer rank
  int32_t* wcnt = seg + E + 1;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int b = blockIdx.x;
  // this lane's tokens (wave-contiguous), fetched first so that the loads overlap the prefix work below
  const int wbase = b * kDispatchTokensPerBlock + wave * kTokPerWave;
  int my_e[kIter], my_p[kIter];
#pragma unroll
  for (int k = 0; k < kIter; ++k) {
    const int m = wbase + k * kWave + lane;
    my_e[k] = m < T ? eid[m] : -1;
  }

  // tokens per expert in earlier blocks, and in all blocks: thread (rg, e) adds the rows q = rg, rg+R, ...
  // of the [blocks, E] count matrix (independent loads), then the R partials are added in order
  {
    const int R = E < kDispThreads ? kDispThreads / E : 1;  // row groups working on one chunk of experts
    int32_t* part_before = wcnt;                             // [R][E] scratch (wcnt is zeroed afterwards)
    int32_t* part_all = wcnt + kDispThreads;                 // R*E <= kDispThreads when R > 1
    for (int e0 = 0; e0 < E; e0 += kDispThreads) {
      const int e = e0 + (R > 1 ? tid % E : tid), rg = R > 1 ? tid / E : 0;
      int before = 0, all = 0;
      if (e < E && rg < R && rg < nblocks) {
        // (unconditional loads - rows past the end re-read row rg and are not added - so that a batch of eight is
        // in flight at once; with the bound inside the loop every load waited for the one before it)
        for (int q0 = rg; q0 < nblocks; q0 += 8 * R) {
          int c[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int q = q0 + u * R;
            c[u] = blockcnt[(size_t)(q < nblocks ? q : rg) * E + e];
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int q = q0 + u * R;
            before += q < b ? c[u] : 0;   // (b < nblocks: rows past the end are never before this block)
            all += q < nblocks ? c[u] : 0;
          }
        }
      }
      if (R > 1) {
        if (rg < R) { part_before[rg * E + e] = before; part_all[rg * E + e] = all; }
        __syncthreads();
        if (tid < E) {
          before = 0; all = 0;
          for (int q = 0; q < R; ++q) { before += part_before[q * E + tid]; all += part_all[q * E + tid]; }
        }
        __syncthreads();
      }
      const int eo = R > 1 ? tid : e;
      if (eo < E && (R == 1 || tid < E)) {
        off[eo] = before;
        tot[eo] = all < C ? all : C;  // kept[e] = min(cnt[e], C)
        node[eo] = e2n ? e2n[eo] : eo / (E / N);
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < kDispWaves * E; i += kDispThreads) wcnt[i] = 0;
  __syncthreads();
  // buffer order: experts sorted by (node, id)
  for (int e = tid; e < E; e += kDispThreads) {
    int r = e;
    if (e2n) {
      r = 0;
      const int ne = node[e];
      for (int q = 0; q < E; ++q) r += (node[q] < ne || (node[q] == ne && q < e)) ? 1 : 0;
    }
    rank[e] = r;
    seg[r + 1] = tot[e];  // staged: kept of the expert at rank r, scanned below
  }
  __syncthreads();
  if (wave == 0) {  // inclusive scan of seg[1..E] by one wave: lane owns a contiguous run
    const int per = ceil_div(E, kWave);
    const int lo = lane * per, hi = min(E, lo + per);
    int s = 0;
    for (int i = lo; i < hi; ++i) s += seg[i + 1];
    int incl = s;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int o = __shfl_up(incl, d);
      if (lane >= d) incl += o;
    }
    int run = incl - s;
    if (lane == 0) seg[0] = 0;
    for (int i = lo; i < hi; ++i) {
      run += seg[i + 1];
      seg[i + 1] = run;
    }
  }
  __syncthreads();
  if (b == 0) {
    for (int e = tid; e < E; e += kDispThreads) {
      kept[e] = tot[e];
      buf_expert[rank[e]] = e;
    }
    for (int i = tid; i <= E; i += kDispThreads) seg_off[i] = seg[i];
    // node nu starts where its first expert starts: the number of kept rows on lower nodes
    for (int nu = tid; nu <= N; nu += kDispThreads) {
      int s = 0;
      for (int e = 0; e < E; ++e) s += node[e] < nu ? tot[e] : 0;
      node_off[nu] = s;
    }
  }

  // rank of each token among the block's earlier tokens of the same expert
  int32_t* wc = wcnt + wave * E;
#pragma unroll
  for (int k = 0; k < kIter; ++k) {
    const bool valid = my_e[k] >= 0;
    const int e = valid ? my_e[k] : 0;
    unsigned long long peers = __ballot(valid);
    for (int bit = 0; bit < nbits; ++bit) {
      const bool set = (e >> bit) & 1;
      const unsigned long long bm = __ballot(valid && set);
      peers &= set ? bm : ~bm;
    }
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int before = __popcll(peers & lt);
    int p = 0;
    if (valid) p = wc[e] + before;       // all lanes read the wave's running count ...
    wave_sync();
    if (valid && before == 0) wc[e] = p + __popcll(peers);  // ... then each group's first lane advances it
    wave_sync();
    my_p[k] = p;
  }
  __syncthreads();
  // ordered prefix over the block's waves (in place: wcnt[w][e] := tokens of e in waves < w)
  for (int e = tid; e < E; e += kDispThreads) {
    int run = off[e];
#pragma unroll
    for (int q = 0; q < kDispWaves; ++q) {
      const int c = wcnt[q * E + e];
      wcnt[q * E + e] = run;
      run += c;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kIter; ++k) {
    const int m = wbase + k * kWave + lane;
    const int e = my_e[k];
    if (e >= 0) {
      const int p = wc[e] + my_p[k];
      pos[m] = p;
      int s = -1;
      if (p < C) {
        s = seg[rank[e]] + p;
        row_token[s] = m;
      }
      slot[m] = s;
    }
  }
}

// send[r,:] = x[row_token[r],:].  A row is `chunks` 16-byte vectors; LPR lanes share a row.  Blocks walk the
// K kept rows with a grid stride; the token index of the next row is fetched before the current row is
// copied, so the index -> row dependency is off the critical path.
constexpr int kCopyBlocksPerCu = 8;

template <int LPR>
__global__ __launch_bounds__(kDispThreads) void dispatch_copy_kernel(const uint4* __restrict__ x,
                                                                     const int32_t* __restrict__ row_token,
                                                                     const int32_t* __restrict__ seg_off,
                                                                     uint4* __restrict__ send, int E, int chunks) {
  constexpr int RPB = kDispThreads / LPR;
  constexpr int U = 4;
  const int K = seg_off[E];
  const int l = threadIdx.x % LPR;
  const int stride = gridDim.x * RPB;
  int r = blockIdx.x * RPB + threadIdx.x / LPR;
  int tok = r < K ? row_token[r] : 0;
  while (r < K) {
    const int rn = r + stride;
    const int tokn = rn < K ? row_token[rn] : 0;
    const uint4* src = x + (size_t)tok * chunks;
    uint4* dst = send + (size_t)r * chunks;
    int c = l;
    for (; c + (U - 1) * LPR < chunks; c += U * LPR) {
      uint4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = nt_load16(src + c + u * LPR);
#pragma unroll
      for (int u = 0; u < U; ++u) dst[c + u * LPR] = v[u];  // plain stores: the FFN re-reads send right away
    }
    for (; c < chunks; c += LPR) dst[c] = nt_load16(src + c);
    r = rn;
    tok = tokn;
  }
}

template <int LPR>
void launch_copy(const void* x, const int32_t* row_token, const int32_t* seg_off, void* send, int E, int rows,
                 int chunks, hipStream_t st) {
  constexpr int RPB = kDispThreads / LPR;
  const int blocks = min(ceil_div(rows, RPB), cu_count() * kCopyBlocksPerCu);
  hipLaunchKernelGGL((dispatch_copy_kernel<LPR>), dim3(blocks), dim3(kDispThreads), 0, st, (const uint4*)x,
                     row_token, seg_off, (uint4*)send, E, chunks);
}


// The three launches of the dispatch; `blockcnt` holds ceil(T/1024) x E counts (every one is written by the first
// kernel before the second reads it: nothing has to be cleared).
int dispatch_launch(const locmoe_desc* desc, const void* x, const int32_t* eid, const int32_t* e2n, int32_t* pos,
                    int32_t* slot, int32_t* kept, int32_t* seg_off, int32_t* node_off, int32_t* buf_expert,
                    int32_t* row_token, void* send, int32_t* blockcnt, hipStream_t s) {
  const int T = desc->T, E = desc->E;
  const int nblocks = ceil_div(T, kDispatchTokensPerBlock);
  hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nblocks), dim3(kDispThreads), (size_t)E * 4, s, eid, blockcnt, T,
                     E);
  int st = launch_status();
  if (st != LOCMOE_OK) return st;
  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  const size_t wcnt_ints = (size_t)kDispWaves * E > 2 * (size_t)kDispThreads ? (size_t)kDispWaves * E : 2 * (size_t)kDispThreads;
  const size_t smem = ((size_t)E * 5 + 1 + wcnt_ints) * 4;
  hipLaunchKernelGGL(dispatch_slots_kernel, dim3(nblocks), dim3(kDispThreads), smem, s, eid, e2n, blockcnt, pos,
                     slot, kept, seg_off, node_off, buf_expert, row_token, T, E, desc->N, desc->C, nblocks, nbits);
  st = launch_status();
  if (st != LOCMOE_OK) return st;
  // at most min(T, E*C) rows can be kept; the kernel reads the real K from seg_off[E]
  const long long cap = (long long)E * desc->C;
  const int rows = (int)(cap < T ? cap : T);
  const int chunks = desc->d * (desc->x_dtype == LOCMOE_BF16 ? 2 : 4) / 16;
  // lanes per row: every lane should own at least 4 chunks so that 4 loads are in flight before the stores
  if (chunks >= 1024) launch_copy<256>(x, row_token, seg_off, send, E, rows, chunks, s);
  else if (chunks >= 512) launch_copy<128>(x, row_token, seg_off, send, E, rows, chunks, s);
  else if (chunks >= 256) launch_copy<64>(x, row_token, seg_off, send, E, rows, chunks, s);
  else if (chunks >= 128) launch_copy<32>(x, row_token, seg_off, send, E, rows, chunks, s);
  else if (chunks >= 64) launch_copy<16>(x, row_token, seg_off, send, E, rows, chunks, s);
  else launch_copy<8>(x, row_token, seg_off, send, E, rows, chunks, s);
  return launch_status();
}

int dispatch_check(const locmoe_desc* desc, const void* x, const int32_t* eid, const int32_t* e2n, int32_t* pos,
                   int32_t* slot, int32_t* kept, int32_t* seg_off, int32_t* node_off, int32_t* buf_expert,
                   int32_t* row_token, void* send) {
  if (!desc || !x || !eid || !pos || !slot || !kept || !seg_off || !node_off || !buf_expert || !row_token ||
      !send)
    return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  if (!e2n && desc->E % desc->N != 0) return LOCMOE_ERR_SHAPE;
  return LOCMOE_OK;
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_dispatch(const locmoe_desc* desc, const void* x, const int32_t* eid, const int32_t* e2n,
                               int32_t* pos, int32_t* slot, int32_t* kept, int32_t* seg_off, int32_t* node_off,
                               int32_t* buf_expert, int32_t* row_token, void* send, void* ws, size_t ws_bytes,
                               void* stream) {
  using namespace locmoe;
  const int st = dispatch_check(desc, x, eid, e2n, pos, slot, kept, seg_off, node_off, buf_expert, row_token, send);
  if (st != LOCMOE_OK) return st;
  if (!ws || ws_bytes < locmoe_workspace_bytes(desc)) return LOCMOE_ERR_WORKSPACE;
  return dispatch_launch(desc, x, eid, e2n, pos, slot, kept, seg_off, node_off, buf_expert, row_token, send,
                         (int32_t*)ws, as_stream(stream));
}

// For callers that cannot allocate: locmoe_dispatch with the count matrix in the library's static scratch.
extern "C" int locmoe_dispatch_static(const locmoe_desc* desc, const void* x, const int32_t* eid, const int32_t* e2n,
                                      int32_t* pos, int32_t* slot, int32_t* kept, int32_t* seg_off,
                                      int32_t* node_off, int32_t* buf_expert, int32_t* row_token, void* send,
                                      void* stream) {
  using namespace locmoe;
  const int st = dispatch_check(desc, x, eid, e2n, pos, slot, kept, seg_off, node_off, buf_expert, row_token, send);
  if (st != LOCMOE_OK) return st;
  const size_t counts = (size_t)ceil_div(desc->T, kDispatchTokensPerBlock) * (size_t)desc->E;
  if (counts * sizeof(int32_t) > kStaticScratchBytes) return LOCMOE_ERR_WORKSPACE;  // beyond the stated maximum
  void* ptr = static_scratch();
  if (!ptr) return LOCMOE_ERR_HIP;
  return dispatch_launch(desc, x, eid, e2n, pos, slot, kept, seg_off, node_off, buf_expert, row_token, send,
                         (int32_t*)ptr, as_stream(stream));
}
