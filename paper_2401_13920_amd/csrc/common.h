// Internal helpers shared by the gfx950 kernels of liblocmoe (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "locmoe.h"

namespace locmoe {

constexpr int kWave = 64;  // CDNA wavefront width

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// 16-byte streaming accesses (non-temporal hint: the data is touched once by this kernel)
__device__ __forceinline__ uint4 nt_load16(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store16(const uint4& v, uint4* p) {
  u32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, (u32x4*)p);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Round-to-nearest-even float -> bf16 bits (finite inputs); gfx950 has the conversion in hardware.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
// two floats -> two bf16 in one register (one v_cvt_pk_bf16_f32), lo in bits 0..15
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  const bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// Sum of the 8 bf16 values held in a 16-byte vector, as a fixed fp32 tree.
__device__ __forceinline__ float sum8_bf16(const uint4& v) {
  float a0 = bf16_bits_to_f32(v.x & 0xFFFFu), a1 = __uint_as_float(v.x & 0xFFFF0000u);
  float a2 = bf16_bits_to_f32(v.y & 0xFFFFu), a3 = __uint_as_float(v.y & 0xFFFF0000u);
  float a4 = bf16_bits_to_f32(v.z & 0xFFFFu), a5 = __uint_as_float(v.z & 0xFFFF0000u);
  float a6 = bf16_bits_to_f32(v.w & 0xFFFFu), a7 = __uint_as_float(v.w & 0xFFFF0000u);
  return ((a0 + a1) + (a2 + a3)) + ((a4 + a5) + (a6 + a7));
}
__device__ __forceinline__ float sum4_f32(const uint4& v) {
  return (__uint_as_float(v.x) + __uint_as_float(v.y)) + (__uint_as_float(v.z) + __uint_as_float(v.w));
}
// the same trees over the squares
__device__ __forceinline__ float sumsq8_bf16(const uint4& v) {
  float a0 = bf16_bits_to_f32(v.x & 0xFFFFu), a1 = __uint_as_float(v.x & 0xFFFF0000u);
  float a2 = bf16_bits_to_f32(v.y & 0xFFFFu), a3 = __uint_as_float(v.y & 0xFFFF0000u);
  float a4 = bf16_bits_to_f32(v.z & 0xFFFFu), a5 = __uint_as_float(v.z & 0xFFFF0000u);
  float a6 = bf16_bits_to_f32(v.w & 0xFFFFu), a7 = __uint_as_float(v.w & 0xFFFF0000u);
  return ((a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3)) + ((a4 * a4 + a5 * a5) + (a6 * a6 + a7 * a7));
}
__device__ __forceinline__ float sumsq4_f32(const uint4& v) {
  const float a = __uint_as_float(v.x), b = __uint_as_float(v.y), c = __uint_as_float(v.z), d = __uint_as_float(v.w);
  return (a * a + b * b) + (c * c + d * d);
}

// v * w for the 4 fp32 or 8 bf16 values of a 16-byte vector (products in fp32, rounded to the storage type)
template <bool BF16>
__device__ __forceinline__ uint4 scale16(const uint4& v, float w) {
  uint4 r;
  if (BF16) {
    const uint32_t* p = &v.x;
    uint32_t* q = &r.x;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      q[i] = pack_bf16x2(w * bf16_bits_to_f32(p[i] & 0xFFFFu), w * __uint_as_float(p[i] & 0xFFFF0000u));
  } else {
    r.x = __float_as_uint(w * __uint_as_float(v.x));
    r.y = __float_as_uint(w * __uint_as_float(v.y));
    r.z = __float_as_uint(w * __uint_as_float(v.z));
    r.w = __float_as_uint(w * __uint_as_float(v.w));
  }
  return r;
}

// ---- cross-lane moves on the DPP path (no LDS traffic) ------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each group of 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside each row of 16

// All-reduce sum over aligned groups of L lanes (L a power of two <= 64): every lane of a
// group ends with the group's total.  The steps below 16 lanes are DPP; 16 and 32 go through
// the cross-lane permute unit.  The order of additions is fixed, so the result is deterministic.
template <int L>
__device__ __forceinline__ float group_sum(float v) {
  if (L >= 2) v += dpp_f32<kDppXor1>(v);
  if (L >= 4) v += dpp_f32<kDppXor2>(v);
  if (L >= 8) v += dpp_f32<kDppHalfMirror>(v);
  if (L >= 16) v += dpp_f32<kDppMirror>(v);
  if (L >= 32) v += __shfl_xor(v, 16);
  if (L >= 64) v += __shfl_xor(v, 32);
  return v;
}

// ---- direct global -> LDS copies -------------------------------------------------------------
typedef const char __attribute__((address_space(3))) * lds_cptr;

// One wave-wide 1 KiB copy global -> LDS: lane l reads 16 bytes at sbase + voff and they land at
// LDS byte address lds_base + 16 l (M0 carries the wave-uniform LDS base).  Default cache policy: nt, sc1
// and sc0 sc1 on the weight stream all measured equal or slower.
__device__ __forceinline__ void dma_1k(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase),
               "s"(lds_base)
               : "memory", "m0");
}
// The same copy in two parts, for runs of copies whose LDS destinations lie within 4 KiB of a common base: M0 is
// written once (dma_base) and each copy adds an immediate offset of sub KiB (dma_1k_sub).  The hardware adds the
// immediate to the LDS address and to the global address alike (M0 + imm + 16 l and sbase + voff + imm), so
// callers whose source does not advance in step with the destination take it off voff.  Nothing else in the
// calling loop may write M0 between the two parts (the compiler only does so for instructions these kernels do
// not use; their listings are checked).
__device__ __forceinline__ void dma_base(uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(lds_base) : "memory", "m0");
}
__device__ __forceinline__ void dma_1k_sub(const void* sbase, uint32_t voff, int sub) {
  switch (sub) {
    case 0: asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase) : "memory"); break;
    case 1: asm volatile("global_load_lds_dwordx4 %0, %1 offset:1024" ::"v"(voff), "s"(sbase) : "memory"); break;
    case 2: asm volatile("global_load_lds_dwordx4 %0, %1 offset:2048" ::"v"(voff), "s"(sbase) : "memory"); break;
    default: asm volatile("global_load_lds_dwordx4 %0, %1 offset:3072" ::"v"(voff), "s"(sbase) : "memory"); break;
  }
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__host__ __device__ constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline int launch_status() { return hipGetLastError() == hipSuccess ? LOCMOE_OK : LOCMOE_ERR_HIP; }

// host-side validation shared by the entry points
int check_desc(const locmoe_desc* d);
// compute units of the current device (the grid of the persistent kernels), 256 if the query fails; asked once
// per device
int cu_count();

// Raises a kernel's dynamic-LDS limit to `bytes`, once per device: `done` (one per kernel) remembers the devices
// it has been raised on, so that the launch path of later calls holds no runtime call beyond the launch itself.
inline bool allow_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  const bool known = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64;
  if (known && ((done.load(std::memory_order_relaxed) >> dev) & 1u)) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
  if (known) done.fetch_or(uint64_t(1) << dev, std::memory_order_relaxed);
  return true;
}

// route / dispatch scratch layout (see workspace.cpp)
constexpr int kRouteMaxBlocks = 512;     // upper bound of route blocks (partials per block)
constexpr int kDispatchTokensPerBlock = 1024;

}  // namespace locmoe
