// Weight gradients of Eq. 1's two linear maps, per expert segment of the send buffer:
//   dW_out[e] = dout_e^T . H_e   ([d,h]),   dW_in[e] = dZ_e^T . send_e   ([h,d])
// i.e. G[e][m][n] = sum over the segment's rows r of P[r][m] * Q[r][n].  Both operands are stored with the
// contracted axis (the rows) outermost, the opposite of what an MFMA lane wants (8 consecutive k for one
// m or n).  gfx950's transposing LDS read (ds_read_b64_tr_b16) delivers exactly that from a k-major tile:
// within 16 lanes, lane i receives element i%4 of the 8-byte groups addressed by lanes i/4, i/4+4, i/4+8,
// i/4+12, so when lane s addresses row k0 + s/4, columns c0 + 4 (s%4).., lane i ends up with column c0 + i
// of rows k0..k0+3.
// The contraction is short (a segment has at most C rows) and the output is large (E d h values per weight):
// at the paper's shapes the kernel is bound by writing G, not by the MFMAs.
#include <algorithm>

#include "common.h"

namespace locmoe {
namespace {

constexpr int kWgTile = 256;              // output tile: 256 (m) x 256 (n)
constexpr int kWgK = 32;                  // rows of the segment per step
constexpr int kWgThreads = 256;           // four waves, each 128 x 128 of the tile
constexpr int kWgRowBytes = kWgTile * 2 + 32;   // 544 B: consecutive rows start 8 banks apart, so the four rows
                                                // that a 16-lane group of the transposing read touches cover all
                                                // 32 banks once
constexpr int kWgSide = kWgK * kWgRowBytes;     // one operand tile of one stage
constexpr int kWgSmem = 4 * kWgSide;            // two stages x two operands

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

__device__ __forceinline__ bf16x8 read_tr8(const char __attribute__((address_space(3))) * p) {
  // rows k0..k0+3 and k0+4..k0+7 of one column: two transposing reads, 4 * kWgRowBytes apart
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
  const s16x4 hi =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 4 * kWgRowBytes));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// grid: E * (Mdim/256) * (Ndim/256) tiles, segment-major, the m-tiles of one n-tile adjacent.
__global__ __launch_bounds__(kWgThreads) void wgrad_256_kernel(const uint16_t* __restrict__ P,
                                                               const uint16_t* __restrict__ Q,
                                                               uint16_t* __restrict__ G,
                                                               const int32_t* __restrict__ seg_off,
                                                               const int32_t* __restrict__ buf_expert, int Mdim,
                                                               int Ndim) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int MT = Mdim / kWgTile, NT = Ndim / kWgTile;
  const int tpe = MT * NT;
  const int r = blockIdx.x / tpe, within = blockIdx.x % tpe;
  const int mt = within % MT, nt = within / MT;
  const int seg0 = seg_off[r], rows = seg_off[r + 1] - seg0;
  const int e = buf_expert[r];
  const int wm = wave >> 1, wn = wave & 1;
  const int kq = lane >> 4, l16 = lane & 15;
  uint16_t* Gt = G + ((size_t)e * Mdim + (size_t)mt * kWgTile) * Ndim + (size_t)nt * kWgTile;

  f32x4 acc[8][8];  // [n subtile][m subtile]: D[n][m], a lane holds n = 4 kq .. +3 for m = l16
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (rows > 0) {
    // staging: thread t copies chunks t, t+256, t+512, t+768 of each operand tile (32 rows x 32 chunks of 16 B)
    const int srow = tid >> 5, scol = tid & 31;  // rows srow, srow+8, srow+16, srow+24
    const uint16_t* Pp = P + (size_t)seg0 * Mdim + (size_t)mt * kWgTile + scol * 8;
    const uint16_t* Qp = Q + (size_t)seg0 * Ndim + (size_t)nt * kWgTile + scol * 8;
    uint4 rp[4], rq[4];
    auto fetch = [&](int k0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // rows past the segment's end belong to the next expert: they are read clamped and replaced by zeros
        const int k = k0 + srow + 8 * i;
        const int kc = min(k, rows - 1);
        const uint4 vp = *(const uint4*)(Pp + (size_t)kc * Mdim);
        const uint4 vq = *(const uint4*)(Qp + (size_t)kc * Ndim);
        rp[i] = k < rows ? vp : make_uint4(0, 0, 0, 0);
        rq[i] = k < rows ? vq : make_uint4(0, 0, 0, 0);
      }
    };
    auto stash = [&](int stage) {
      char* base = smem + stage * 2 * kWgSide;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int off = (srow + 8 * i) * kWgRowBytes + scol * 16;
        *(uint4*)(base + off) = rp[i];
        *(uint4*)(base + kWgSide + off) = rq[i];
      }
    };
    const char __attribute__((address_space(3)))* lds =
        (const char __attribute__((address_space(3)))*)(uintptr_t)(uint32_t)(uintptr_t)(
            __attribute__((address_space(3))) char*)smem;
    // this lane's address inside an operand tile for subtile 0: row 8 kq + l16/4, column 4 (l16 % 4)
    const int lane_off = (8 * kq + (l16 >> 2)) * kWgRowBytes + (l16 & 3) * 8;
    const int steps = (rows + kWgK - 1) / kWgK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int ks = 0; ks < steps; ++ks) {
      const int stage = ks & 1;
      if (ks + 1 < steps) fetch((ks + 1) * kWgK);
      const char __attribute__((address_space(3)))* pt = lds + stage * 2 * kWgSide + lane_off;
      bf16x8 fm[8], fn[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) fm[j] = read_tr8(pt + (wm * 128 + j * 16) * 2);
#pragma unroll
      for (int j = 0; j < 8; ++j) fn[j] = read_tr8(pt + kWgSide + (wn * 128 + j * 16) * 2);
#pragma unroll
      for (int ni = 0; ni < 8; ++ni)
#pragma unroll
        for (int mj = 0; mj < 8; ++mj)
          acc[ni][mj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fn[ni], fm[mj], acc[ni][mj], 0, 0, 0);
      if (ks + 1 < steps) stash(stage ^ 1);
      __syncthreads();
    }
  }
  // an expert without rows gets zeros: every element of G is written
#pragma unroll
  for (int mj = 0; mj < 8; ++mj) {
    const int m = wm * 128 + mj * 16 + l16;
#pragma unroll
    for (int ni = 0; ni < 8; ++ni) {
      const int n = wn * 128 + ni * 16 + kq * 4;
      const f32x4 v = acc[ni][mj];
      *(uint2*)(Gt + (size_t)m * Ndim + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Pipelined form for the paper's shapes.  One work-group per compute unit walks through its tiles; the operand
// tiles of the next three k-steps (of this tile or the next) are always in flight as direct global->LDS copies
// into a ring of four stages, so the short contraction (at most C rows: 16 steps at C = 501) never starts
// cold.  Only those copies are outstanding while a tile is computed, so they retire in order and a counted
// wait tells when a step's data has landed; the tile's stores are drained (vmcnt(0)) before the next tile's
// waits count again.  LDS rows are 512 B with the 16-byte chunk index XORed by 2 (row mod 4): the four rows
// that a 16-lane group of the transposing read touches then start 8 banks apart.
// Rows past the segment's end are read clamped (finite duplicates of the last row) and the P side's copies of
// them are overwritten with zeros by the wave that fetched them, so their products vanish.
// Tiles: XCD x (work-groups x mod 8) owns a contiguous eighth of the segment-major tile list, so an expert's
// operands live in one L2; inside a segment, 32 consecutive tiles (the XCD's work-groups at one time) form a
// block of 4 m-tiles x 8 n-tiles (12 operand tiles for 32 outputs).  Segments without rows are skipped here
// and zero-filled by wgrad_zero_empty_kernel.
constexpr int kWgStages = 4;
constexpr int kWgSideBytes = kWgK * kWgTile * 2;   // 16 KiB
constexpr int kWgStageBytes = 2 * kWgSideBytes;    // P tile, then Q tile
constexpr int kWgDmaSmem = kWgStages * kWgStageBytes;

struct WgTile {          // wave-uniform
  const char* P;         // the segment's first row at the tile's first m column
  const char* Q;         // ... n column
  uint16_t* G;           // the output tile's origin
  int rows;              // rows of the segment (> 0)
};

__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char*)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ bf16x8 read_tr8_sw(lds_cptr p) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 4 * 512));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

__global__ __launch_bounds__(kWgThreads) void wgrad_dma_kernel(const uint16_t* __restrict__ P,
                                                               const uint16_t* __restrict__ Q,
                                                               uint16_t* __restrict__ G,
                                                               const int32_t* __restrict__ seg_off,
                                                               const int32_t* __restrict__ buf_expert, int Mdim,
                                                               int Ndim, int E) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int MT = Mdim / kWgTile, NT = Ndim / kWgTile;
  const int tpe = MT * NT;
  const int total = E * tpe;
  const int nwg = gridDim.x;
  const bool blocked = (MT % 4 == 0) && (NT % 8 == 0);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  lds_cptr lds = (lds_cptr)(uintptr_t)lds0;

  // tile number t of the launch (t mod 8 = XCD) -> position in the segment-major list
  auto tile_of = [&](int t, int& rows_out) -> WgTile {
    const int u = (total % 8 == 0) ? (t & 7) * (total >> 3) + (t >> 3) : t;
    const int r = u / tpe, within = u - r * tpe;
    int mt, nt;
    if (blocked) {
      const int b = within >> 5, i = within & 31, mb = MT >> 2;
      mt = (b % mb) * 4 + (i & 3);
      nt = (b / mb) * 8 + (i >> 2);
    } else {
      mt = within % MT;
      nt = within / MT;
    }
    const int seg0 = seg_off[r];
    rows_out = seg_off[r + 1] - seg0;
    WgTile w;
    w.rows = rows_out;
    w.P = uniform_ptr((const char*)(P + (size_t)seg0 * Mdim + (size_t)mt * kWgTile));
    w.Q = uniform_ptr((const char*)(Q + (size_t)seg0 * Ndim + (size_t)nt * kWgTile));
    w.G = G + ((size_t)buf_expert[r] * Mdim + (size_t)mt * kWgTile) * Ndim + (size_t)nt * kWgTile;
    return w;
  };
  // the first tile at or after t (in this work-group's sequence) whose segment has rows
  auto next_live = [&](int t, WgTile& w) -> int {
    while (t < total) {
      int rows;
      w = tile_of(t, rows);
      if (rows > 0) break;
      t += nwg;
    }
    return __builtin_amdgcn_readfirstlane(t);
  };

  WgTile cur;
  int t_cur = next_live(blockIdx.x, cur);
  if (t_cur >= total) return;

  // ---- the copy side: a cursor three steps ahead of the compute side
  WgTile pf = cur;
  int t_pf = t_cur, k_pf = 0, stage_pf = 0;
  bool pf_live = true;
  const int half = lane >> 5, ch = lane & 31;
  const uint32_t ldP = (uint32_t)Mdim * 2, ldQ = (uint32_t)Ndim * 2;
  auto issue = [&]() -> bool {
    if (!pf_live) return false;
    const uint32_t sbase = lds0 + (uint32_t)stage_pf * kWgStageBytes + (uint32_t)wave * 8 * 512;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = 8 * wave + 2 * q + half;              // row of the k-step that this lane copies
      const int kc = min(k_pf + r, pf.rows - 1);          // clamped: always a row of this segment
      const uint32_t chunk = (uint32_t)(ch ^ (((2 * q + half) & 3) << 1));
      dma_1k(pf.P, (uint32_t)kc * ldP + chunk * 16, sbase + q * 1024);
      dma_1k(pf.Q, (uint32_t)kc * ldQ + chunk * 16, sbase + kWgSideBytes + q * 1024);
    }
    stage_pf = (stage_pf + 1) & (kWgStages - 1);
    k_pf += kWgK;
    if (k_pf >= pf.rows) {
      t_pf = next_live(t_pf + nwg, pf);
      pf_live = t_pf < total;
      k_pf = 0;
    }
    return true;
  };
  int ahead = 0;  // steps issued and not yet computed
#pragma unroll
  for (int i = 0; i < kWgStages - 1; ++i) ahead += issue() ? 1 : 0;

  // ---- the compute side
  const int wm = wave >> 1, wn = wave & 1;
  const int kq = lane >> 4, l16 = lane & 15;
  const int rr = l16 >> 2;
  int off_m[8], off_n[8];  // this lane's byte offsets inside a P / Q tile for its eight subtiles
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int lo = (8 * kq + rr) * 512 + ((l16 & 3) >> 1) * 16 + (l16 & 1) * 8;
    off_m[j] = lo + (16 * wm + 2 * (j ^ rr)) * 16;
    off_n[j] = lo + (16 * wn + 2 * (j ^ rr)) * 16 + kWgSideBytes;
  }
  int stage = 0;
  for (;;) {
    f32x4 acc[8][8];  // [n subtile][m subtile]: D[n][m], a lane holds n = 4 kq .. +3 for m = l16
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int steps = (cur.rows + kWgK - 1) / kWgK;
    for (int s = 0; s < steps; ++s) {
      // this step's copies have landed when at most the younger ones (8 per step and wave) are outstanding
      if (ahead >= 3) wait_vmcnt<16>();
      else if (ahead == 2) wait_vmcnt<8>();
      else wait_vmcnt<0>();
      const int rem = cur.rows - s * kWgK;  // live rows of this step
      if (rem < kWgK) {
        char* pt = smem + stage * kWgStageBytes;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int r = 8 * wave + 2 * q + half;
          if (r >= rem) *(uint4*)(pt + r * 512 + ch * 16) = make_uint4(0, 0, 0, 0);
        }
      }
      __syncthreads();
      ahead += issue() ? 1 : 0;  // into the stage that was read one step ago
      lds_cptr pt = lds + stage * kWgStageBytes;
      bf16x8 fm[8], fn[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) fm[j] = read_tr8_sw(pt + off_m[j]);
#pragma unroll
      for (int j = 0; j < 8; ++j) fn[j] = read_tr8_sw(pt + off_n[j]);
#pragma unroll
      for (int ni = 0; ni < 8; ++ni)
#pragma unroll
        for (int mj = 0; mj < 8; ++mj)
          acc[ni][mj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fn[ni], fm[mj], acc[ni][mj], 0, 0, 0);
      --ahead;
      stage = (stage + 1) & (kWgStages - 1);
    }
    uint16_t* Gt = cur.G;
#pragma unroll
    for (int mj = 0; mj < 8; ++mj) {
      const int m = wm * 128 + mj * 16 + l16;
#pragma unroll
      for (int ni = 0; ni < 8; ++ni) {
        const int n = wn * 128 + ni * 16 + kq * 4;
        const f32x4 v = acc[ni][mj];
        *(uint2*)(Gt + (size_t)m * Ndim + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
      }
    }
    wait_vmcnt<0>();  // the stores must not be in flight when the next tile's waits count copies
    t_cur = next_live(t_cur + nwg, cur);
    if (t_cur >= total) break;
  }
}

// G[e] = 0 for experts whose segment has no rows (the pipelined kernel skips them)
__global__ __launch_bounds__(256) void wgrad_zero_empty_kernel(uint4* __restrict__ G,
                                                               const int32_t* __restrict__ seg_off,
                                                               const int32_t* __restrict__ buf_expert,
                                                               size_t chunks_per_expert) {
  const int r = blockIdx.y;
  if (seg_off[r + 1] != seg_off[r]) return;
  uint4* g = G + (size_t)buf_expert[r] * chunks_per_expert;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < chunks_per_expert; i += (size_t)gridDim.x * 256)
    g[i] = make_uint4(0, 0, 0, 0);
}

// Any shape: one thread per output element, the segment's rows in order.  Correct, not tuned.
template <bool P_F32, bool Q_F32>
__global__ __launch_bounds__(256) void wgrad_generic_kernel(const void* __restrict__ P, const void* __restrict__ Q,
                                                            uint16_t* __restrict__ G,
                                                            const int32_t* __restrict__ seg_off,
                                                            const int32_t* __restrict__ buf_expert, int Mdim,
                                                            int Ndim) {
  const int r = blockIdx.z;
  const int n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int m = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (n >= Ndim || m >= Mdim) return;
  const int seg0 = seg_off[r], rows = seg_off[r + 1] - seg0;
  float s = 0.f;
  for (int k = 0; k < rows; ++k) {
    const size_t row = (size_t)seg0 + k;
    const float p = P_F32 ? ((const float*)P)[row * Mdim + m] : bf16_bits_to_f32(((const uint16_t*)P)[row * Mdim + m]);
    const float q = Q_F32 ? ((const float*)Q)[row * Ndim + n] : bf16_bits_to_f32(((const uint16_t*)Q)[row * Ndim + n]);
    s = fmaf(p, q, s);
  }
  G[((size_t)buf_expert[r] * Mdim + m) * Ndim + n] = f32_to_bf16_bits(s);
}

inline int wg_cu_count() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8)
    return 256;
  return n;
}

template <bool P_F32, bool Q_F32>
int launch_wgrad(const void* P, const void* Q, void* G, const int32_t* seg_off, const int32_t* buf_expert, int E,
                 int rows_max, int Mdim, int Ndim, hipStream_t st) {
  if (!P_F32 && !Q_F32 && Mdim % kWgTile == 0 && Ndim % kWgTile == 0) {
    const long long total = (long long)E * (Mdim / kWgTile) * (Ndim / kWgTile);
    const long long span = (long long)rows_max * (Mdim > Ndim ? Mdim : Ndim) * 2;  // byte offsets inside a segment
    if (total <= 0x3FFFFFFFLL && span < 0x7FFFFFFFLL) {
      if (hipFuncSetAttribute((const void*)wgrad_dma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                              kWgDmaSmem) != hipSuccess)
        return LOCMOE_ERR_HIP;
      const size_t chunks = (size_t)Mdim * Ndim / 8;
      hipLaunchKernelGGL(wgrad_zero_empty_kernel, dim3(64, E), dim3(256), 0, st, (uint4*)G, seg_off, buf_expert,
                         chunks);
      const long long groups = std::min<long long>((wg_cu_count() / 8) * 8, (total + 7) / 8 * 8);
      hipLaunchKernelGGL(wgrad_dma_kernel, dim3((unsigned)groups), dim3(kWgThreads), kWgDmaSmem, st,
                         (const uint16_t*)P, (const uint16_t*)Q, (uint16_t*)G, seg_off, buf_expert, Mdim, Ndim, E);
      return launch_status();
    }
    if (total <= 0x7FFFFFFFLL) {
      if (hipFuncSetAttribute((const void*)wgrad_256_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kWgSmem) !=
          hipSuccess)
        return LOCMOE_ERR_HIP;
      hipLaunchKernelGGL(wgrad_256_kernel, dim3((unsigned)total), dim3(kWgThreads), kWgSmem, st, (const uint16_t*)P,
                         (const uint16_t*)Q, (uint16_t*)G, seg_off, buf_expert, Mdim, Ndim);
      return launch_status();
    }
  }
  if (ceil_div(Mdim, 4) > 65535 || E > 65535) return LOCMOE_ERR_SHAPE;
  hipLaunchKernelGGL((wgrad_generic_kernel<P_F32, Q_F32>), dim3(ceil_div(Ndim, 64), ceil_div(Mdim, 4), E), dim3(256),
                     0, st, P, Q, (uint16_t*)G, seg_off, buf_expert, Mdim, Ndim);
  return launch_status();
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_expert_ffn_wgrad(const locmoe_desc* desc, const void* send, const void* H, const void* dout,
                                       const void* dZ, const int32_t* seg_off, const int32_t* buf_expert,
                                       void* dW_in, void* dW_out, void* stream) {
  using namespace locmoe;
  if (!desc || !send || !H || !dout || !dZ || !seg_off || !buf_expert || !dW_in || !dW_out) return LOCMOE_ERR_NULL;
  int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  hipStream_t s = as_stream(stream);
  const int E = desc->E, d = desc->d, h = desc->h;
  const int rows_max = desc->C < desc->T ? desc->C : desc->T;
  if (desc->x_dtype == LOCMOE_F32) {
    st = launch_wgrad<false, true>(dZ, send, dW_in, seg_off, buf_expert, E, rows_max, h, d, s);   // dW_in[e] = dZ^T . send
    if (st != LOCMOE_OK) return st;
    return launch_wgrad<true, false>(dout, H, dW_out, seg_off, buf_expert, E, rows_max, d, h, s);  // dW_out[e] = dout^T . H
  }
  st = launch_wgrad<false, false>(dZ, send, dW_in, seg_off, buf_expert, E, rows_max, h, d, s);
  if (st != LOCMOE_OK) return st;
  return launch_wgrad<false, false>(dout, H, dW_out, seg_off, buf_expert, E, rows_max, d, h, s);
}
