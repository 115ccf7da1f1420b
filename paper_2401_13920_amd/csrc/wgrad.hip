// Weight gradients of Eq. 1's two linear maps, per expert segment of the send buffer:
//   dW_out[e] = dout_e^T . H_e   ([d,h]),   dW_in[e] = dZ_e^T . send_e   ([h,d])
// i.e. G[e][m][n] = sum over the segment's rows r of P[r][m] * Q[r][n].  Both operands are stored with the
// contracted axis (the rows) outermost, the opposite of what an MFMA lane wants (8 consecutive k for one
// m or n).  gfx950's transposing LDS read (ds_read_b64_tr_b16) delivers exactly that from a k-major tile:
// within 16 lanes, lane i receives element i%4 of the 8-byte groups addressed by lanes i/4, i/4+4, i/4+8,
// i/4+12, so when lane s addresses row k0 + s/4, columns c0 + 4 (s%4).., lane i ends up with column c0 + i
// of rows k0..k0+3.
// The contraction is short (a segment has at most C rows) and the output is large (E d h values per weight):
// at the paper's headline shape writing G takes a quarter of the kernel's time (measured by leaving the stores
// out), the rest is the MFMA loop at the rate of the forward GEMMs.
#include <algorithm>

#include "common.h"

namespace locmoe {
namespace {

constexpr int kWgTile = 256;              // output tile: 256 (m) x 256 (n)
constexpr int kWgK = 32;                  // rows of the segment per step
constexpr int kWgThreads = 256;           // four waves, each 128 x 128 of the tile

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// MFMA kernel for shapes whose d and h are multiples of 256 (the paper's).  One work-group per compute unit
// walks through its tiles; the operand tiles of the next three k-steps (of this tile or the next) are always in flight as direct global->LDS copies
// into a ring of four stages, so the short contraction (at most C rows: 16 steps at C = 501) never starts
// cold.  Copies complete in issue order among themselves, so a counted wait (as many as were issued after the
// step's own) tells when a step's data has landed, also with the previous tile's stores still in flight.
// LDS rows are 512 B with the 16-byte chunk index XORed by 2 s(row), s = row mod 4 plus
// 4 (bit 3 of the row): the eight rows that 32 lanes of the transposing read touch (rows r..r+3 and r+8..r+11,
// 32 B each) then fall into all 64 banks once; with row mod 4 alone half of the LDS cycles were bank conflicts.
// Rows past the segment's end are read clamped (finite duplicates of the last row) and the P side's copies of
// them are overwritten with zeros by the wave that fetched them, so their products vanish.
// Tiles: XCD x (work-groups x mod 8) owns whole segments, so an expert's operands live in one L2; inside a
// segment, 32 consecutive tiles (the XCD's work-groups at one time) form a block of 4 m-tiles x 8 n-tiles
// (12 operand tiles for 32 outputs).  Segments without rows are skipped here and zero-filled by
// wgrad_zero_empty_kernel.
constexpr int kWgQBytes = kWgK * kWgTile * 2;   // the Q tile of a step: 32 rows x 256 columns, 16 KiB

struct WgShape {
  static constexpr int kMJ = 8;                    // 16-row m-subtiles per wave: a wave owns 128 x 128 of the tile
  static constexpr int kTM = 2 * kMJ * 16;         // tile rows (m): 256
  static constexpr int kPRow = kTM * 2;            // bytes of a P row in LDS
  static constexpr int kPBytes = kWgK * kPRow;
  static constexpr int kStage = kPBytes + kWgQBytes;
  static constexpr int kStages = 4;
  static constexpr int kSmem = kStages * kStage;   // 128 KiB: one work-group per compute unit
  static constexpr int kPLanes = kPRow / 16;       // lanes per P row in a copy
  static constexpr int kPRowsPerCopy = 64 / kPLanes;
  static constexpr int kPCopies = 8 / kPRowsPerCopy;      // per wave and step (a wave copies 8 of the 32 rows)
  static constexpr int kCopies = kPCopies + 4;            // ... plus four for the Q tile
};

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

// rows k0..k0+3 and k0+4..k0+7 of one column: two transposing reads, four LDS rows apart
template <int ROW_BYTES>
__device__ __forceinline__ bf16x8 read_tr8_sw(lds_cptr p) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
  const s16x4 hi =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 4 * ROW_BYTES));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

__global__ __launch_bounds__(kWgThreads) void wgrad_dma_kernel(
    const uint16_t* __restrict__ P, const uint16_t* __restrict__ Q, uint16_t* __restrict__ G,
    const int32_t* __restrict__ seg_off, const int32_t* __restrict__ buf_expert, int Mdim, int Ndim, int E) {
  using S = WgShape;
  constexpr int MJ = S::kMJ;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int MT = Mdim / S::kTM, NT = Ndim / kWgTile;
  const int tpe = MT * NT;
  const int total = E * tpe;
  const int nwg = gridDim.x;
  // work-groups that run side by side on an XCD take a block of MB x 8 tiles of one segment
  constexpr int MB = 4;
  const bool blocked = (MT % MB == 0) && (NT % 8 == 0);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  lds_cptr lds = (lds_cptr)(uintptr_t)lds0;

  // Which segments an XCD owns.  With E a multiple of 8 the segments are ranked by descending row count and
  // dealt to the XCDs in boustrophedon order (ranks 0..7 to XCDs 0..7, ranks 8..15 to XCDs 7..0, ...): every
  // XCD gets E/8 segments with nearly the same number of rows, largest first (the headline input: 16 % more
  // steps on the busiest XCD with contiguous eighths of the buffer order, 1 % this way).  Otherwise tile t
  // simply is tile t of the segment-major list.
  __shared__ int32_t s_tab[128];  // segment of this XCD's local rank k
  const bool ranked = (E & 7) == 0;
  if (ranked) {
    int32_t* s_seg = (int32_t*)smem;  // [E+1], before the ring is in use
    for (int t = tid; t <= E; t += kWgThreads) s_seg[t] = seg_off[t];
    __syncthreads();
    const int xcd = blockIdx.x & 7;
    for (int t = tid; t < E; t += kWgThreads) {
      const int mine = s_seg[t + 1] - s_seg[t];
      int rank = 0;
      for (int q = 0; q < E; ++q) {
        const int other = s_seg[q + 1] - s_seg[q];
        rank += (other > mine || (other == mine && q < t)) ? 1 : 0;
      }
      const int deal = rank >> 3, pos = rank & 7;
      if (((deal & 1) ? 7 - pos : pos) == xcd) s_tab[deal] = t;
    }
    __syncthreads();  // the table is complete and nobody reads the staging area any more
  }

  // tile number t of the launch (t mod 8 = XCD) -> segment and position inside it
  auto tile_of = [&](int t, int& rows_out) -> WgTile {
    int r, within;
    if (ranked) {
      const int j = t >> 3, k = j / tpe;  // the XCD's j-th tile lies in its k-th segment
      r = __builtin_amdgcn_readfirstlane(s_tab[k]);
      within = j - k * tpe;
    } else {
      r = t / tpe;
      within = t - r * tpe;
    }
    int mt, nt;
    if (blocked) {
      const int b = within / (MB * 8), i = within % (MB * 8), mb = MT / MB;
      mt = (b % mb) * MB + (i % MB);
      nt = (b / mb) * 8 + (i / MB);
    } else {
      mt = within % MT;
      nt = within / MT;
    }
    const int seg0 = seg_off[r];
    rows_out = seg_off[r + 1] - seg0;
    WgTile w;
    w.rows = rows_out;
    w.P = uniform_ptr((const char*)(P + (size_t)seg0 * Mdim + (size_t)mt * S::kTM));
    w.Q = uniform_ptr((const char*)(Q + (size_t)seg0 * Ndim + (size_t)nt * kWgTile));
    w.G = G + ((size_t)buf_expert[r] * Mdim + (size_t)mt * S::kTM) * Ndim + (size_t)nt * kWgTile;
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

  // ---- the copy side: a cursor kStages - 1 steps ahead of the compute side
  WgTile pf = cur;
  int t_pf = t_cur, k_pf = 0, stage_pf = 0;
  bool pf_live = true;
  const int prow = lane / S::kPLanes, pch = lane % S::kPLanes;  // P copies: row inside the copy, chunk
  const int qrow = lane >> 5, qch = lane & 31;                  // Q copies
  const uint32_t ldP = (uint32_t)Mdim * 2, ldQ = (uint32_t)Ndim * 2;
  const int swz_hi = (wave & 1) << 2;  // bit 3 of the rows this wave copies (rows 8 wave .. 8 wave + 7)
  // What a copy's source offset is made of, per lane and copy, computed once: the row's byte offset inside a step
  // and the (swizzled) chunk.  A step then costs an add, a min (rows past the segment's end re-read its last row)
  // and an add per copy instead of a multiplication and the swizzle arithmetic: with one wave per SIMD every
  // instruction between two MFMAs is MFMA time (the copies' address arithmetic was 1.1 ms of the 8.3 ms of both
  // GEMMs at config 4).  The four copies of an operand land in consecutive KiB of LDS: one M0 write serves them,
  // each copy carries its KiB as immediate offset, which the hardware also adds to the source address; it is taken
  // off the chunk term again (from a base 4 KiB below the operand, so that the offset stays non-negative).
  static_assert(S::kPCopies == 4 && S::kPRowsPerCopy == 2, "the copy tables assume 512-byte P rows");
  uint32_t rowP[4], chP[4], rowQ[4], chQ[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r8p = 2 * q + prow, r8q = 2 * q + qrow;  // row inside the wave's eight
    rowP[q] = (uint32_t)(8 * wave + r8p) * ldP;
    chP[q] = (uint32_t)(pch ^ (((r8p & 3) | swz_hi) << 1)) * 16 + 4096 - q * 1024;
    rowQ[q] = (uint32_t)(8 * wave + r8q) * ldQ;
    chQ[q] = (uint32_t)(qch ^ (((r8q & 3) | swz_hi) << 1)) * 16 + 4096 - q * 1024;
  }
  auto issue = [&]() -> bool {
    if (!pf_live) return false;
    const uint32_t sbase = lds0 + (uint32_t)stage_pf * S::kStage;
    const uint32_t kP = (uint32_t)k_pf * ldP, kQ = (uint32_t)k_pf * ldQ;                     // this step's first row
    const uint32_t endP = (uint32_t)(pf.rows - 1) * ldP, endQ = (uint32_t)(pf.rows - 1) * ldQ;  // the segment's last row
    dma_base(sbase + (uint32_t)wave * 8 * S::kPRow);
#pragma unroll
    for (int q = 0; q < 4; ++q) dma_1k_sub(pf.P - 4096, min(rowP[q] + kP, endP) + chP[q], q);
    dma_base(sbase + S::kPBytes + (uint32_t)wave * 4096);
#pragma unroll
    for (int q = 0; q < 4; ++q) dma_1k_sub(pf.Q - 4096, min(rowQ[q] + kQ, endQ) + chQ[q], q);
    stage_pf = stage_pf + 1 == S::kStages ? 0 : stage_pf + 1;
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
  for (int i = 0; i < S::kStages - 1; ++i) ahead += issue() ? 1 : 0;

  // ---- the compute side
  const int wm = wave >> 1, wn = wave & 1;
  const int kq = lane >> 4, l16 = lane & 15;
  const int sw = (l16 >> 2) | ((kq & 1) << 2);  // the swizzle of the rows this lane addresses
  int off_m[MJ], off_n[8];  // this lane's byte offsets inside a stage for its subtiles
  {
    const int row = 8 * kq + (l16 >> 2), b1 = (l16 & 3) >> 1, inner = (l16 & 1) * 8;
#pragma unroll
    for (int j = 0; j < MJ; ++j) off_m[j] = row * S::kPRow + (((2 * MJ * wm + 2 * j + b1) ^ (sw << 1)) << 4) + inner;
#pragma unroll
    for (int j = 0; j < 8; ++j) off_n[j] = S::kPBytes + row * 512 + (((16 * wn + 2 * j + b1) ^ (sw << 1)) << 4) + inner;
  }
  int stage = 0, stage_last = 0;
  for (;;) {
    f32x4 acc[8][MJ];  // [n subtile][m subtile]: D[n][m], a lane holds n = 4 kq .. +3 for m = l16
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int b = 0; b < MJ; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int steps = (cur.rows + kWgK - 1) / kWgK;
    for (int s = 0; s < steps; ++s) {
      // this step's copies have landed when at most the younger ones (kCopies per step and wave) are outstanding
      if (ahead >= S::kStages - 1) wait_vmcnt<(S::kStages - 2) * S::kCopies>();
      else if (ahead == 2) wait_vmcnt<S::kCopies>();
      else wait_vmcnt<0>();
      const int rem = cur.rows - s * kWgK;  // live rows of this step
      if (rem < kWgK) {
        char* pt = smem + stage * S::kStage + wave * 8 * S::kPRow;
#pragma unroll
        for (int q = 0; q < S::kPCopies; ++q) {
          const int r8 = S::kPRowsPerCopy * q + prow;
          if (8 * wave + r8 >= rem) *(uint4*)(pt + r8 * S::kPRow + pch * 16) = make_uint4(0, 0, 0, 0);
        }
      }
      __syncthreads();
      ahead += issue() ? 1 : 0;  // into the stage that was read one step ago
      lds_cptr pt = lds + stage * S::kStage;
      bf16x8 fm[MJ], fn[8];
#pragma unroll
      for (int j = 0; j < MJ; ++j) fm[j] = read_tr8_sw<S::kPRow>(pt + off_m[j]);
#pragma unroll
      for (int j = 0; j < 8; ++j) fn[j] = read_tr8_sw<512>(pt + off_n[j]);
#pragma unroll
      for (int ni = 0; ni < 8; ++ni)
#pragma unroll
        for (int mj = 0; mj < MJ; ++mj)
          acc[ni][mj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fn[ni], fm[mj], acc[ni][mj], 0, 0, 0);
      --ahead;
      stage_last = stage;
      stage = stage + 1 == S::kStages ? 0 : stage + 1;
    }
    // Epilogue through LDS: a lane holds 4 consecutive n of one row m, which stored directly are 8-byte
    // pieces in 32-byte runs (measured: 1.5 TB/s, twice the time of the MFMAs).  Each wave turns one 16-row
    // subtile at a time into rows of 256 contiguous bytes in its quarter of the stage that the last step
    // read (free until the next step's copies) and stores 16 bytes per lane, four whole rows per instruction.
    // Two 4 KiB buffers alternate, so a subtile is written while the previous one is read back; the 16-byte
    // chunk index is XORed with the row, which spreads both the 8-byte writes of 32 lanes (16 rows x 2 column
    // groups) and the 16-byte reads of 16 lanes (one row) over all 64 banks.
    __syncthreads();  // every wave has finished reading that stage
    {
      char* mine = smem + stage_last * S::kStage + wave * (S::kStage / 4);
      uint16_t* Gw = cur.G + (size_t)(wm * (MJ * 16)) * Ndim + wn * 128;
      const int rrow = lane >> 4, rcol = lane & 15;
      auto put = [&](int mj) {
        char* buf = mine + (mj & 1) * 4096 + l16 * 256 + (kq & 1) * 8;
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) {
          const f32x4 v = acc[ni][mj];
          *(uint2*)(buf + (((2 * ni + (kq >> 1)) ^ l16) << 4)) =
              make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        }
      };
      put(0);
#pragma unroll
      for (int mj = 0; mj < MJ; ++mj) {
        if (mj + 1 < MJ) put(mj + 1);
        const char* buf = mine + (mj & 1) * 4096;
#pragma unroll
        for (int p4 = 0; p4 < 4; ++p4) {
          const int row = 4 * p4 + rrow;
          const uint4 v = *(const uint4*)(buf + row * 256 + ((rcol ^ row) << 4));
          nt_store16(v, (uint4*)(Gw + (size_t)(mj * 16 + row) * Ndim + rcol * 8));  // written once, read by nobody here
        }
      }
    }
    // No drain of the stores: the waits above stay sufficient with stores in flight.  Copies complete in issue
    // order among themselves, so while a step's copy is outstanding so are all younger copies, and the counter
    // exceeds their number whatever the stores do; stores only make a wait last longer.
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

template <bool P_F32, bool Q_F32>
int launch_wgrad(const void* P, const void* Q, void* G, const int32_t* seg_off, const int32_t* buf_expert, int E,
                 int rows_max, int Mdim, int Ndim, hipStream_t st) {
  if (!P_F32 && !Q_F32 && Mdim % kWgTile == 0 && Ndim % kWgTile == 0) {
    const long long total = (long long)E * (Mdim / kWgTile) * (Ndim / kWgTile);
    const long long span = (long long)rows_max * (Mdim > Ndim ? Mdim : Ndim) * 2;  // byte offsets inside a segment
    if (total <= 0x3FFFFFFFLL && span < 0x7FFFFFFFLL) {
      using S = WgShape;
      auto kern = wgrad_dma_kernel;
      static std::atomic<uint64_t> lds_allowed;
      if (!allow_lds((const void*)kern, S::kSmem, lds_allowed)) return LOCMOE_ERR_HIP;
      const size_t chunks = (size_t)Mdim * Ndim / 8;
      hipLaunchKernelGGL(wgrad_zero_empty_kernel, dim3(64, E), dim3(256), 0, st, (uint4*)G, seg_off, buf_expert,
                         chunks);
      const long long tiles = (long long)E * (Mdim / S::kTM) * (Ndim / kWgTile);
      const long long groups = std::min<long long>((cu_count() / 8) * 8, (tiles + 7) / 8 * 8);
      hipLaunchKernelGGL(kern, dim3((unsigned)groups), dim3(kWgThreads), S::kSmem, st, (const uint16_t*)P,
                         (const uint16_t*)Q, (uint16_t*)G, seg_off, buf_expert, Mdim, Ndim, E);
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
