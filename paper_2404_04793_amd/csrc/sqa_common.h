// Internal helpers shared by the HIP translation units of libsqa (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <map>
#include <mutex>
#include <utility>
#include "sqa.h"

#define SQA_WAVE 64

namespace sqa {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

struct bf16_t { uint16_t bits; };          // storage tag for SQA_BF16

template <typename T> struct elem;
template <> struct elem<float>  { static constexpr int per16 = 4; };
template <> struct elem<bf16_t> { static constexpr int per16 = 8; };

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (inputs are finite here; NaN kept quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// c + a.lo*b.lo + a.hi*b.hi on two packed bf16 pairs (v_dot2_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// 16-byte global-memory accesses.  Every pointer the kernels get is device
// global memory, but many arrive through a struct read from memory, which the
// compiler can only treat as generic ("flat"); flat loads also count against the
// LDS wait counter, which would serialise them with LDS traffic.  Hence the
// explicit global address space.
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) v4u_t g_v4u_t;
__device__ __forceinline__ uint4 ld16(const void* p) {
  const v4u_t v = *(const g_v4u_t*)(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
// marked non-temporal (global_load_dwordx4 ... nt): data that is streamed once
// per launch.  On MI355X a pure streaming read reaches about 7.1 TB/s with nt
// loads against about 6.3 TB/s with plain loads.
__device__ __forceinline__ uint4 ld16_nt(const void* p) {
  const v4u_t v = __builtin_nontemporal_load((const g_v4u_t*)(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16(void* p, uint4 v) {
  *(g_v4u_t*)(p) = v4u_t{v.x, v.y, v.z, v.w};
}

template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, SQA_WAVE);
  return v;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// A kernel needs a one-time opt-in per device before a launch may ask for more dynamic LDS than the
// default limit.  Remembered per (device, kernel), so the steady state makes no runtime call for it and a
// caller that records launches into a HIP graph only has to run each kernel once eagerly before.
inline hipError_t allow_dynamic_lds(const void* fn, size_t bytes) {
  static std::mutex mu;
  static std::map<std::pair<int, const void*>, size_t> granted;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  size_t& g = granted[std::make_pair(dev, fn)];
  if (g >= bytes) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) g = bytes;
  return e;
}

#define SQA_HIP_CHECK(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return SQA_ERR_HIP; } } while (0)

}  // namespace sqa
