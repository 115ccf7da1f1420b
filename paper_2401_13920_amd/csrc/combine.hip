// Gate-weighted combine (Eq. 1 with the top-1 score of Eq. 3): y[m,:] = w[m] * out[slot[m],:]
// for kept tokens, zeros for dropped ones.  With top-1 routing every y row has exactly one
// contribution, so each row is written once: no adds, no atomics.  Bandwidth-bound.
#include "common.h"

namespace locmoe {
namespace {

constexpr int kCombThreads = 256;

// LPR lanes share one token row of `chunks` 16-byte vectors; one block per group of rows.  Measured at the
// headline shape (8 KiB rows): many lanes per row with one or two chunks each beats fewer lanes with deeper
// unrolling, and a grid-stride loop is slower than one short-lived block per row group.
template <bool BF16, int LPR>
__global__ __launch_bounds__(kCombThreads) void combine_kernel(const uint4* __restrict__ out,
                                                               const int32_t* __restrict__ slot,
                                                               const float* __restrict__ w, uint4* __restrict__ y,
                                                               int T, int chunks) {
  constexpr int RPB = kCombThreads / LPR;
  const int m = blockIdx.x * RPB + threadIdx.x / LPR;
  if (m >= T) return;
  const int l = threadIdx.x % LPR;
  const int s = slot[m];
  uint4* dst = y + (size_t)m * chunks;
  if (s < 0) {
    for (int c = l; c < chunks; c += LPR) nt_store16(make_uint4(0, 0, 0, 0), dst + c);
    return;
  }
  const float wm = w[m];
  const uint4* src = out + (size_t)s * chunks;
  constexpr int U = 4;
  int c = l;
  for (; c + (U - 1) * LPR < chunks; c += U * LPR) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = nt_load16(src + c + u * LPR);
#pragma unroll
    for (int u = 0; u < U; ++u) nt_store16(scale16<BF16>(v[u], wm), dst + c + u * LPR);
  }
  for (; c < chunks; c += LPR) nt_store16(scale16<BF16>(nt_load16(src + c), wm), dst + c);
}

template <bool BF16, int LPR>
void launch(const void* out, const int32_t* slot, const float* w, void* y, int T, int chunks, hipStream_t st) {
  constexpr int RPB = kCombThreads / LPR;
  hipLaunchKernelGGL((combine_kernel<BF16, LPR>), dim3(ceil_div(T, RPB)), dim3(kCombThreads), 0, st,
                     (const uint4*)out, slot, w, (uint4*)y, T, chunks);
}

template <bool BF16>
void dispatch_lpr(const void* out, const int32_t* slot, const float* w, void* y, int T, int chunks,
                  hipStream_t st) {
  if (chunks >= 256) launch<BF16, 256>(out, slot, w, y, T, chunks, st);
  else if (chunks >= 128) launch<BF16, 128>(out, slot, w, y, T, chunks, st);
  else if (chunks >= 64) launch<BF16, 64>(out, slot, w, y, T, chunks, st);
  else if (chunks >= 32) launch<BF16, 32>(out, slot, w, y, T, chunks, st);
  else if (chunks >= 16) launch<BF16, 16>(out, slot, w, y, T, chunks, st);
  else launch<BF16, 8>(out, slot, w, y, T, chunks, st);
}

}  // namespace
}  // namespace locmoe

extern "C" int locmoe_combine(const locmoe_desc* desc, const void* out, const int32_t* slot, const float* w,
                              void* y, void* stream) {
  using namespace locmoe;
  if (!desc || !out || !slot || !w || !y) return LOCMOE_ERR_NULL;
  const int st = check_desc(desc);
  if (st != LOCMOE_OK) return st;
  const bool bf = desc->x_dtype == LOCMOE_BF16;
  const int chunks = desc->d * (bf ? 2 : 4) / 16;
  if (bf) dispatch_lpr<true>(out, slot, w, y, desc->T, chunks, as_stream(stream));
  else dispatch_lpr<false>(out, slot, w, y, desc->T, chunks, as_stream(stream));
  return launch_status();
}
