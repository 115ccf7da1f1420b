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
                 int Mdim, int Ndim, hipStream_t st) {
  if (!P_F32 && !Q_F32 && Mdim % kWgTile == 0 && Ndim % kWgTile == 0) {
    const long long total = (long long)E * (Mdim / kWgTile) * (Ndim / kWgTile);
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
  if (desc->x_dtype == LOCMOE_F32) {
    st = launch_wgrad<false, true>(dZ, send, dW_in, seg_off, buf_expert, E, h, d, s);   // dW_in[e] = dZ^T . send
    if (st != LOCMOE_OK) return st;
    return launch_wgrad<true, false>(dout, H, dW_out, seg_off, buf_expert, E, d, h, s);  // dW_out[e] = dout^T . H
  }
  st = launch_wgrad<false, false>(dZ, send, dW_in, seg_off, buf_expert, E, h, d, s);
  if (st != LOCMOE_OK) return st;
  return launch_wgrad<false, false>(dout, H, dW_out, seg_off, buf_expert, E, d, h, s);
}
